// bfloat16 tree attention on the matrix cores (head dimension 128).
//
// One workgroup = 4 waves = up to 256 query rows of one (sequence, KV head, key split); every wave
// owns 64 rows (two 32-row MFMA column blocks) and keeps their output accumulators in registers for
// the whole pass, so K and V are read from HBM once per workgroup and shared through LDS by all
// G x M rows of the KV head (Section 2.2: every tree row attends to the same prefix).
//
// Both products are computed transposed with v_mfma_f32_32x32x16_bf16:
//     S^T[key, row] = K[key, :] . Q[row, :]      A = K fragment (LDS), B = Q fragment (registers)
//     O^T[d,  row] += V^T[d, key] P^T[key, row]  A = V fragment (LDS), B = P (registers)
// In the S^T accumulator a lane holds 16 keys of ONE row, so the softmax maximum and sum are
// in-lane reductions plus one exchange between the two half-waves, and P^T is already laid out as
// the B operand of the second product: no transposition of P through LDS.  The contraction order of
// the keys inside a 16-key MFMA step is permuted to match that layout; V fragments are fetched with
// the same permutation.  The output dimension is permuted as d = 4 * i + t (t = 32-row block of
// O^T, i = row inside it) so that a lane fetches the four blocks' values of one key with a single
// 8-byte LDS read and writes 4 consecutive output elements at the end.
//
// Softmax runs in the log2 domain with a lazily updated reference maximum: accumulators are only
// rescaled when a new score exceeds the reference by more than 2^8, which is exact after the final
// division by the (equally referenced) denominator.
// The tree part (ancestor mask) is a bit table built in LDS from the parent pointers.
//
// K/V tiles go from HBM straight into LDS (global_load_lds_dwordx4, 16 bytes per lane, no staging
// registers) through a ring of four tile buffers, three tiles ahead of the one being multiplied, so
// about 96 KB per compute unit are in flight.  The XOR swizzle that keeps LDS reads conflict-free
// is applied on the global side: the lane that fills LDS slot c of a row fetches chunk c ^ (row & 7).
// Waits are explicit (s_waitcnt vmcnt(n) counts this wave's younger tile loads) and the workgroup
// barrier carries no memory fence, so outstanding loads survive it.
#include "attn_common.h"

namespace hs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* glb_ptr;

#ifndef HS_ABL
#define HS_ABL 9
#endif
constexpr int MF_ROWS = 256;     // query rows per workgroup (64 per wave)
constexpr int MF_TILE = 64;      // keys per LDS tile
constexpr int MF_NBUF = 4;       // LDS ring: one tile being multiplied, three on their way from HBM
constexpr int MF_MAX_M = 256;    // tree rows per sequence (ancestor bit table: M x 8 words)
constexpr int MF_ROW_BYTES = 256;  // one K or V row of a head: 128 bf16
constexpr int MF_TILE_BYTES = MF_TILE * MF_ROW_BYTES;
constexpr float MF_LOG2E = 1.4426950408889634f;
constexpr float MF_LN2 = 0.6931471805599453f;
constexpr float MF_LAZY = 8.0f;  // rescale only when the reference maximum is exceeded by 2^8

bool attn_mfma_supported(int D, hs_dtype dt, int max_tree_rows, float scale) {
  return D == 128 && dt == HS_BF16 && max_tree_rows <= MF_MAX_M && scale > 0.f;
}

// 16-byte chunk c (0..15) of row r lives at chunk position c ^ (r & 7): conflict-free for both the
// row-per-lane K reads and the row-per-half-wave V reads.
__device__ __forceinline__ int swz(int row, int chunk) { return row * MF_ROW_BYTES + ((chunk ^ (row & 7)) << 4); }

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_addr + 16 i.
// lds_addr is a wave-uniform LDS byte address (placed in M0).
__device__ __forceinline__ void lds_dma16(const char* gptr, unsigned lds_addr) {
  const unsigned m = __builtin_amdgcn_readfirstlane(lds_addr);
  unsigned saved;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
      : "=&s"(saved)
      : "s"(m), "v"(gptr)
      : "memory");
}

struct TileSrc {
  const char* k;
  const char* v;
  int64_t base;   // first key of the tile (token index in the prefix, or tree row)
  int64_t limit;  // keys at or beyond it do not exist
  bool tree;
};

// QT = 32-row blocks per wave: 2 -> 4 waves of 64 rows, 1 -> 8 waves of 32 rows (two waves per SIMD,
// so one wave's softmax arithmetic overlaps the other's matrix instructions).
template <int QT>
__global__ __launch_bounds__(512 / QT) void k_attn_mfma(AttnArgs a, int n_rg_max) {
  constexpr int THREADS = 512 / QT;
  constexpr int LOADS = 1024 / THREADS;  // 16-byte chunks of K (and of V) per thread per tile
  __shared__ __attribute__((aligned(16))) char lds_k[MF_NBUF][MF_TILE_BYTES];
  __shared__ __attribute__((aligned(16))) char lds_v[MF_NBUF][MF_TILE_BYTES];
  __shared__ unsigned anc[MF_MAX_M * 8];

  const int s = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int n0 = a.node_offsets[s];
  const int M = a.node_offsets[s + 1] - n0;
  const int64_t p0 = a.prefix_offsets[s];
  const int64_t L = a.prefix_offsets[s + 1] - p0;
  if (M <= 0) return;
  const int G = a.G, Hkv = a.Hkv, Hq = a.Hq;
  const int R = G * M;
  const int n_rg = (R + MF_ROWS - 1) / MF_ROWS;
  const int n_sp = splits_of(L, a.split_len);
  int x = blockIdx.x;
  const int g = x % Hkv;
  x /= Hkv;
  const int rg = x % n_rg_max;
  const int sp = x / n_rg_max;
  if (rg >= n_rg || sp >= n_sp) return;

  const char* kp = static_cast<const char*>(a.k_prefix) + (p0 * Hkv + g) * MF_ROW_BYTES;
  const char* vp = static_cast<const char*>(a.v_prefix) + (p0 * Hkv + g) * MF_ROW_BYTES;
  const char* kt = static_cast<const char*>(a.k_tree) + ((int64_t)n0 * Hkv + g) * MF_ROW_BYTES;
  const char* vt = static_cast<const char*>(a.v_tree) + ((int64_t)n0 * Hkv + g) * MF_ROW_BYTES;
  const int64_t tok_stride = (int64_t)Hkv * MF_ROW_BYTES;

  const bool last_split = sp == n_sp - 1;
  const int64_t k_lo = (int64_t)sp * a.split_len;
  const int64_t k_hi = last_split ? L : k_lo + a.split_len;
  const int n_ptiles = (int)((k_hi - k_lo + MF_TILE - 1) / MF_TILE);
  const int n_ttiles = last_split ? (M + MF_TILE - 1) / MF_TILE : 0;
  const int n_tiles = n_ptiles + n_ttiles;

  auto tile_src = [&](int t) {
    TileSrc ts;
    ts.tree = t >= n_ptiles;
    if (ts.tree) {
      ts.k = kt; ts.v = vt; ts.base = (int64_t)(t - n_ptiles) * MF_TILE; ts.limit = M;
    } else {
      ts.k = kp; ts.v = vp; ts.base = k_lo + (int64_t)t * MF_TILE; ts.limit = k_hi;
    }
    return ts;
  };

  // ---- ancestor bit table: bit j of row i's words is set iff tree row j is on the root path of i
  if (last_split && tid < M) {
    unsigned w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = tid; j >= 0; j = a.parent[n0 + j]) {
#pragma unroll
      for (int q = 0; q < 8; ++q) w[q] |= ((j >> 5) == q) ? (1u << (j & 31)) : 0u;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) anc[tid * 8 + q] = w[q];
  }

  // ---- this wave's rows and their Q fragments (B operand of the first product)
  const int row_base = rg * MF_ROWS + wave * (32 * QT);
  const bool wave_active = row_base < R;
  bf16x8 qf[QT][8];
  int tree_row[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int r = row_base + qt * 32 + col;
    const int rc = r < R ? r : R - 1;
    const int i = rc / G, gi = rc - i * G;
    tree_row[qt] = i;
    const char* qrow = static_cast<const char*>(a.q) + ((int64_t)(n0 + i) * Hq + g * G + gi) * MF_ROW_BYTES;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[qt][kk] = (r < R && wave_active) ? *reinterpret_cast<const bf16x8*>(qrow + (2 * kk + half) * 16) : z;
    }
  }

  floatx16 acc[QT][4];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt)
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[qt][t][v] = 0.f;
  float m_ref[QT], l_sum[QT];  // log2-domain reference maximum; this lane's share of the denominator
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m_ref[qt] = -HS_INF;
    l_sum[qt] = 0.f;
  }
  const float c2 = a.scale * MF_LOG2E;

  // ---- tile loads: 64 rows x 16 chunks for K and for V; wave w issues rows 4(4j+w) .. +3 of both.
  // Issued as inline assembly: the compiler then neither tracks them in its own wait counters nor
  // orders LDS reads of other ring slots behind them.
  const unsigned lds_k_addr = (unsigned)(uintptr_t)(lds_ptr)&lds_k[0][0];
  const unsigned lds_v_addr = (unsigned)(uintptr_t)(lds_ptr)&lds_v[0][0];
  auto issue = [&](int t) {
    const TileSrc ts = tile_src(t);
    const unsigned ring = (unsigned)(t % MF_NBUF) * MF_TILE_BYTES;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int c = j * THREADS + tid;  // LDS slot (16-byte units) this lane fills
      const int row = c >> 4, slot = c & 15;
      int64_t key = ts.base + row;
      key = key < ts.limit ? key : ts.limit - 1;  // rows past the end repeat the last row (masked later)
      const int64_t off = key * tok_stride + ((slot ^ (row & 7)) << 4);
      const unsigned wave_slot = ring + (unsigned)((j * THREADS + wave * 64) << 4);  // wave-uniform
      lds_dma16(ts.k + off, lds_k_addr + wave_slot);
      lds_dma16(ts.v + off, lds_v_addr + wave_slot);
    }
  };
  if (n_tiles > 0) issue(0);
  if (n_tiles > 1) issue(1);
  if (n_tiles > 2) issue(2);
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // the ancestor table is complete

  // iteration t: wait for tile t, barrier, start the load of tile t+3 into the slot that tile t-1
  // just left, multiply tile t
  for (int t = 0; t < n_tiles; ++t) {
    const TileSrc ts = tile_src(t);
    const char* kb_base = lds_k[t % MF_NBUF];
    const char* vb_base = lds_v[t % MF_NBUF];
    // this wave's loads of tile t are done once at most the 2 x 2 LOADS loads of tiles t+1, t+2 are pending
    if (t + 2 < n_tiles) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(4 * LOADS) : "memory");
    else if (t + 1 < n_tiles) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * LOADS) : "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#ifndef HS_NODMA
    if (t + 3 < n_tiles) issue(t + 3);
#endif
    if (wave_active && HS_ABL >= 1) {
      const bool partial_tile = ts.base + MF_TILE > ts.limit;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        if (ts.base + kb * 32 >= ts.limit) break;  // whole key block beyond the end
        // ---- S^T = K Q^T for 32 keys x 64 rows
        floatx16 sc[QT];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
#pragma unroll
          for (int v = 0; v < 16; ++v) sc[qt][v] = 0.f;
        const int krow = kb * 32 + col;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kb_base + swz(krow, 2 * kk + half));
#pragma unroll
          for (int qt = 0; qt < QT; ++qt)
            sc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qt][kk], sc[qt], 0, 0, 0);
        }
#if HS_ABL == 1
        for (int qt = 0; qt < QT; ++qt) acc[qt][0] += sc[qt];
        continue;
#endif
        // ---- masks: keys past the end of the split; tree keys off the row's root path
        if (ts.tree) {
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) {
            const unsigned word = anc[tree_row[qt] * 8 + (int)((ts.base >> 5) + kb)];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int bit = 8 * (v >> 2) + 4 * half + (v & 3);
              sc[qt][v] = ((word >> bit) & 1u) ? sc[qt][v] : -HS_INF;
            }
          }
        } else if (partial_tile) {
          const int valid = (int)(ts.limit - ts.base) - kb * 32;  // keys of this block that exist
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = 8 * (v >> 2) + 4 * half + (v & 3);
            if (key >= valid) {
#pragma unroll
              for (int qt = 0; qt < QT; ++qt) sc[qt][v] = -HS_INF;
            }
          }
        }
        // ---- softmax numerators in the log2 domain, lazily referenced maximum
        bf16x8 pf[QT][2];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
          float mx = sc[qt][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sc[qt][v]);
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          const float cand = mx * c2;
          const bool grow = cand > m_ref[qt] + MF_LAZY;
          if (__ballot(grow) != 0ull) {
            const float m_new = grow ? cand : m_ref[qt];
            const float alpha = (m_ref[qt] == -HS_INF) ? (grow ? 0.f : 1.f) : exp2_fast(m_ref[qt] - m_new);
            l_sum[qt] *= alpha;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
              for (int v = 0; v < 16; ++v) acc[qt][tt][v] *= alpha;
            m_ref[qt] = m_new;
          }
          float p[16];
          float ps = 0.f;
          const float mr = (m_ref[qt] == -HS_INF) ? 0.f : m_ref[qt];  // (every key masked so far: p = 0)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            p[v] = exp2_fast(fmaf(sc[qt][v], c2, -mr));
            ps += p[v];
          }
          l_sum[qt] += ps;
#pragma unroll
          for (int k2 = 0; k2 < 2; ++k2) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              floatx2 f = {p[8 * k2 + 2 * e], p[8 * k2 + 2 * e + 1]};
              bf16x2 hbits = __builtin_convertvector(f, bf16x2);
              pf[qt][k2][2 * e] = hbits[0];
              pf[qt][k2][2 * e + 1] = hbits[1];
            }
          }
        }
#if HS_ABL == 2
        for (int qt = 0; qt < QT; ++qt) acc[qt][0][0] += (float)pf[qt][0][0] + (float)pf[qt][1][3];
        continue;
#endif
        // ---- O^T += V^T P^T
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          uint2 vfr[8];
#pragma unroll
          for (int idx = 0; idx < 8; ++idx) {
            const int key = kb * 32 + 8 * (2 * k2 + (idx >> 2)) + 4 * half + (idx & 3);
            vfr[idx] = *reinterpret_cast<const uint2*>(vb_base + swz(key, col >> 1) + (col & 1) * 8);
          }
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) {
            unsigned w4[4];
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
              const unsigned lo = (tt < 2) ? vfr[2 * pp].x : vfr[2 * pp].y;
              const unsigned hi = (tt < 2) ? vfr[2 * pp + 1].x : vfr[2 * pp + 1].y;
              w4[pp] = __builtin_amdgcn_perm(hi, lo, (tt & 1) ? 0x07060302u : 0x05040100u);
            }
            uint4 packed = {w4[0], w4[1], w4[2], w4[3]};
            const bf16x8 vf = __builtin_bit_cast(bf16x8, packed);
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
              acc[qt][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qt][k2], acc[qt][tt], 0, 0, 0);
          }
        }
      }
    }
  }

  // ---- results: direct (single split everywhere) or this split's partial record
  if (!wave_active) return;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int r = row_base + qt * 32 + col;
    const float l_tot = l_sum[qt] + __shfl_xor(l_sum[qt], 32);
    if (r >= R) continue;
    const int i = r / G, gi = r - i * G;
    const int64_t row = (int64_t)(n0 + i) * Hq + g * G + gi;
    if (a.sp_max == 1) {
      const float inv = 1.f / l_tot;
      char* out = static_cast<char*>(a.o) + row * MF_ROW_BYTES;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int d0 = 4 * (8 * (v >> 2) + 4 * half + (v & 3));
        floatx2 f01 = {acc[qt][0][v] * inv, acc[qt][1][v] * inv};
        floatx2 f23 = {acc[qt][2][v] * inv, acc[qt][3][v] * inv};
        uint2 pk;
        pk.x = __builtin_bit_cast(unsigned, __builtin_convertvector(f01, bf16x2));
        pk.y = __builtin_bit_cast(unsigned, __builtin_convertvector(f23, bf16x2));
        *reinterpret_cast<uint2*>(out + d0 * 2) = pk;
      }
      if (a.lse && half == 0) a.lse[row] = (m_ref[qt] + __log2f(l_tot)) * MF_LN2;
    } else {
      float* rec = a.part + (row * a.sp_max + sp) * ATTN_REC;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int d0 = 4 * (8 * (v >> 2) + 4 * half + (v & 3));
        float4 f = {acc[qt][0][v], acc[qt][1][v], acc[qt][2][v], acc[qt][3][v]};
        *reinterpret_cast<float4*>(rec + d0) = f;
      }
      if (half == 0) {
        rec[128] = m_ref[qt] * MF_LN2;
        rec[129] = l_tot;
      }
    }
  }
}

#ifndef HS_QT
#define HS_QT 1
#endif
hs_status attn_mfma_launch(const AttnArgs& a, int max_tree_rows, hipStream_t stream) {
  const int n_rg_max = (a.G * max_tree_rows + MF_ROWS - 1) / MF_ROWS;
  dim3 grid((unsigned)(a.Hkv * n_rg_max * a.sp_max), (unsigned)a.B);
  hipLaunchKernelGGL(k_attn_mfma<HS_QT>, grid, dim3(512 / HS_QT), 0, stream, a, n_rg_max);
  return launch_status("tree attention (mfma)");
}

}  // namespace hs
