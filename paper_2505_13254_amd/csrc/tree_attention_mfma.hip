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
#include "attn_common.h"

namespace hs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int MF_THREADS = 256;
constexpr int MF_ROWS = 256;     // query rows per workgroup (64 per wave)
constexpr int MF_TILE = 64;      // keys per LDS tile
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

struct TileSrc {
  const char* k;
  const char* v;
  int64_t base;   // first key of the tile (token index in the prefix, or tree row)
  int64_t limit;  // keys at or beyond it do not exist
  bool tree;
};

__global__ __launch_bounds__(MF_THREADS) void k_attn_mfma(AttnArgs a, int n_rg_max) {
  __shared__ __attribute__((aligned(16))) char lds_k[2][MF_TILE_BYTES];
  __shared__ __attribute__((aligned(16))) char lds_v[2][MF_TILE_BYTES];
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
  const int row_base = rg * MF_ROWS + wave * 64;
  const bool wave_active = row_base < R;
  bf16x8 qf[2][8];
  int tree_row[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
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

  floatx16 acc[2][4];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt)
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[qt][t][v] = 0.f;
  float m_ref[2] = {-HS_INF, -HS_INF};  // log2 domain
  float l_sum[2] = {0.f, 0.f};          // this lane's share of the denominator
  const float c2 = a.scale * MF_LOG2E;

  // ---- staging: 64 rows x 16 chunks for K and for V, four chunks of each per thread
  uint4 kreg[4], vreg[4];
  auto fetch = [&](const TileSrc& ts) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = tid + MF_THREADS * j;
      const int row = c >> 4, ch = c & 15;
      const int64_t key = ts.base + row;
      uint4 z = {0u, 0u, 0u, 0u};
      if (key < ts.limit) {
        kreg[j] = *reinterpret_cast<const uint4*>(ts.k + key * tok_stride + ch * 16);
        vreg[j] = *reinterpret_cast<const uint4*>(ts.v + key * tok_stride + ch * 16);
      } else {
        kreg[j] = z;
        vreg[j] = z;
      }
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = tid + MF_THREADS * j;
      const int row = c >> 4, ch = c & 15;
      *reinterpret_cast<uint4*>(&lds_k[buf][swz(row, ch)]) = kreg[j];
      *reinterpret_cast<uint4*>(&lds_v[buf][swz(row, ch)]) = vreg[j];
    }
  };

  {
    TileSrc ts = tile_src(0);
    fetch(ts);
    stash(0);
  }
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int buf = t & 1;
    const TileSrc ts = tile_src(t);
    if (t + 1 < n_tiles) {
      TileSrc nx = tile_src(t + 1);
      fetch(nx);
    }
    if (wave_active) {
      const char* kb_base = lds_k[buf];
      const char* vb_base = lds_v[buf];
      const bool partial_tile = ts.base + MF_TILE > ts.limit;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        if (ts.base + kb * 32 >= ts.limit) break;  // whole key block beyond the end
        // ---- S^T = K Q^T for 32 keys x 64 rows
        floatx16 sc[2];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          sc[0][v] = 0.f;
          sc[1][v] = 0.f;
        }
        const int krow = kb * 32 + col;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kb_base + swz(krow, 2 * kk + half));
          sc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0][kk], sc[0], 0, 0, 0);
          sc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[1][kk], sc[1], 0, 0, 0);
        }
        // ---- masks: keys past the end of the split; tree keys off the row's root path
        if (ts.tree) {
#pragma unroll
          for (int qt = 0; qt < 2; ++qt) {
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
              sc[0][v] = -HS_INF;
              sc[1][v] = -HS_INF;
            }
          }
        }
        // ---- softmax numerators in the log2 domain, lazily referenced maximum
        bf16x8 pf[2][2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
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
        // ---- O^T += V^T P^T
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          uint2 vr[8];
#pragma unroll
          for (int idx = 0; idx < 8; ++idx) {
            const int key = kb * 32 + 8 * (2 * k2 + (idx >> 2)) + 4 * half + (idx & 3);
            vr[idx] = *reinterpret_cast<const uint2*>(vb_base + swz(key, col >> 1) + (col & 1) * 8);
          }
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) {
            unsigned w4[4];
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
              const unsigned lo = (tt < 2) ? vr[2 * pp].x : vr[2 * pp].y;
              const unsigned hi = (tt < 2) ? vr[2 * pp + 1].x : vr[2 * pp + 1].y;
              w4[pp] = __builtin_amdgcn_perm(hi, lo, (tt & 1) ? 0x07060302u : 0x05040100u);
            }
            uint4 packed = {w4[0], w4[1], w4[2], w4[3]};
            const bf16x8 vf = __builtin_bit_cast(bf16x8, packed);
            acc[0][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[0][k2], acc[0][tt], 0, 0, 0);
            acc[1][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[1][k2], acc[1][tt], 0, 0, 0);
          }
        }
      }
    }
    if (t + 1 < n_tiles) stash(buf ^ 1);
    __syncthreads();
  }

  // ---- results: direct (single split everywhere) or this split's partial record
  if (!wave_active) return;
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
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

hs_status attn_mfma_launch(const AttnArgs& a, int max_tree_rows, hipStream_t stream) {
  const int n_rg_max = (a.G * max_tree_rows + MF_ROWS - 1) / MF_ROWS;
  dim3 grid((unsigned)(a.Hkv * n_rg_max * a.sp_max), (unsigned)a.B);
  hipLaunchKernelGGL(k_attn_mfma, grid, dim3(MF_THREADS), 0, stream, a, n_rg_max);
  return launch_status("tree attention (mfma)");
}

}  // namespace hs
