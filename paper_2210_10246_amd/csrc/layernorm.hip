// In-place LayerNorm for gfx950 (Sec. 3.2; App. D.2, D.3).
//
// Forward: a group of LANES lanes owns one row, held entirely in registers (CH 16-byte pieces
// per lane, piece c of lane t = c*LANES + t), so x is read once; mean and the biased variance are taken in two
// register passes; gamma/beta stay in registers across the rows a group walks.
// Backward: same ownership; xhat is rebuilt from the OUTPUT as (y - beta)/gamma, the two row
// sums are butterfly-reduced, and the column sums for dgamma/dbeta are carried in registers
// across rows, tree-reduced over the workgroup through LDS in a fixed order and written as
// one partial per workgroup; a second small kernel adds the partials in a fixed order.
#include <atomic>
#include <type_traits>

#include "tempo_device.h"
#include "tempo_host.h"

namespace tempo {
namespace {

constexpr int kFwdThreads = 256;
constexpr int kBwdWaves = 8;
constexpr int kBwdThreads = kBwdWaves * kWave;
// Rows of more than 1024 pieces in bfloat16 (8192 columns: 4 pieces per lane of 4 waves) or 2048
// pieces in float32 (8192 columns: 6 or 8 pieces per lane of 4 waves, float32 only, whose pieces
// need half the registers per column) take the generic kernels.  Dynamic LDS of the backward: the column sums' slots (all
// of them, 64*M bytes while a row fits one wave, when that is at most kOneStepLdsBytes; else
// half of them for a tree: 32*M bytes while a row fits one wave, 128 KiB at M = 4096; 16*M over
// two waves; 8*M over four), or gamma, 1/gamma and beta/gamma (12*M bytes, 96 KiB at M = 8192)
// when a lane's share of them does not fit its registers, whichever is more.
constexpr int kMaxFastPieces = 1024;
constexpr int kMaxFastPiecesF32 = 2048;
// Most LDS the backward's column sums may take in one step (every wave's sums at once); two
// workgroups of that size still fit a compute unit.
constexpr size_t kOneStepLdsBytes = 64 * 1024;

// Forward.  A batch is kGroups*R consecutive rows; lane group g takes rows base + r*kGroups + g
// and fetches all R of them (packed) before any arithmetic, so that short rows still keep
// several 16-byte loads per lane in flight.  LOOP = false: one batch per workgroup (the grid
// must cover every batch).  LOOP = true: workgroups walk the batches grid-stride, fetching the
// next batch before they compute on the current one, and load gamma/beta once: for long rows
// the parameters (8 bytes per column from L2) otherwise outweigh the row itself.
template <typename T, int LANES, int CH, int R, bool LOOP>
__global__ __launch_bounds__(kFwdThreads) void ln_fwd_kernel(
    const T* x, const float* __restrict__ gamma, const float* __restrict__ beta, T* y,
    float* __restrict__ rstd_out, float* __restrict__ mean_out, int64_t N, int M, float eps) {
  constexpr int kGroups = kFwdThreads / LANES;
  constexpr int V = Store<T>::kVec;
  const int g = threadIdx.x / LANES;
  const int t = threadIdx.x % LANES;
  const int chunks = M / V;
  // mean and variance by a true division: a row of equal values c then has the mean c exactly
  // (its sum c*M is exact) and zero variance, whatever the rounding of 1/M would do
  const float m_f = static_cast<float>(M);
  __shared__ float red[2][kFwdThreads / kWave];
  static_assert(LANES <= kWave || R == 1, "rows over several waves: one row per group");

  auto fetch = [&](int64_t base, Raw<T> (&f)[R][CH]) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t row = base + r * kGroups + g;
      if (row < N) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const int ch = c * LANES + t;
          if (ch < chunks) f[r][c].load(x + row * M + ch * V);
        }
      }
    }
  };

  int64_t base = static_cast<int64_t>(blockIdx.x) * (kGroups * R);
  if (base >= N) return;  // uniform over the workgroup
  Raw<T> raw[R][CH];
  fetch(base, raw);
  // parameters after the first rows are on their way; they stay in registers for every batch
  float ga[CH][V], be[CH][V];
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    const int ch = c * LANES + t;
    if (ch < chunks) {
      load_floats<V>(gamma + ch * V, ga[c]);
      load_floats<V>(beta + ch * V, be[c]);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i) ga[c][i] = be[c][i] = 0.0f;
    }
  }
  while (true) {
    const int64_t next = base + static_cast<int64_t>(gridDim.x) * (kGroups * R);
    Raw<T> ahead[R][CH];  // unused (and eliminated) without LOOP
    if constexpr (LOOP) {
      if (next < N) fetch(next, ahead);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t row = base + r * kGroups + g;
      // no row: uniform over the lane group; a group of several waves walks on with zeros
      // (the reductions hold workgroup barriers) and stores nothing
      const bool live = row < N;
      if (LANES <= kWave && !live) continue;
      float v[CH][V];
      float sum = 0.0f;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int ch = c * LANES + t;
        if (live && ch < chunks) {
          raw[r][c].unpack(v[c]);
        } else {
#pragma unroll
          for (int i = 0; i < V; ++i) v[c][i] = 0.0f;
        }
#pragma unroll
        for (int i = 0; i < V; ++i) sum += v[c][i];
      }
      const float mu = row_reduce<LANES, false>(sum, red[0]) / m_f;
      float sq = 0.0f;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int ch = c * LANES + t;
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const float d = v[c][i] - mu;
          v[c][i] = d;
          sq += (ch < chunks) ? d * d : 0.0f;
        }
      }
      const float var = row_reduce<LANES, false>(sq, red[1]) / m_f;
      const float rs = 1.0f / sqrtf(var + eps);
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int ch = c * LANES + t;
        if (live && ch < chunks) {
          float o[V];
#pragma unroll
          for (int i = 0; i < V; ++i) o[i] = fmaf(v[c][i] * rs, ga[c][i], be[c][i]);
          store_piece<T>(y + row * M + ch * V, o);
        }
      }
      if (t == 0 && live) {
        rstd_out[row] = rs;
        if (mean_out) mean_out[row] = mu;
      }
    }
    if constexpr (!LOOP) {
      break;
    } else {
      if (next >= N) break;  // uniform over the workgroup
#pragma unroll
      for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int c = 0; c < CH; ++c) raw[r][c] = ahead[r][c];
      }
      base = next;
    }
  }
}

// Sum over a 256-thread workgroup; every thread gets the result.
__device__ __forceinline__ float block_sum_256(float v, float* lds) {
  v = group_sum<kWave>(v);
  const int w = threadIdx.x / kWave;
  lds_barrier();
  if ((threadIdx.x & (kWave - 1)) == 0) lds[w] = v;
  lds_barrier();
  return (lds[0] + lds[1]) + (lds[2] + lds[3]);
}

// Any M: one workgroup per row, scalar accesses.  KC > 0: rows of at most 256 * KC columns, held in
// registers and read once.  KC == 0: any length, x re-read from cache for each pass.
template <typename T, int KC>
__global__ __launch_bounds__(256) void ln_fwd_generic_kernel(
    const T* x, const float* __restrict__ gamma, const float* __restrict__ beta, T* y,
    float* __restrict__ rstd_out, float* __restrict__ mean_out, int64_t N, int64_t M, float eps) {
  __shared__ float lds[4];
  const float m_f = static_cast<float>(M);
  for (int64_t row = blockIdx.x; row < N; row += gridDim.x) {
    const T* xr = x + row * M;
    T* yr = y + row * M;
    float mu, rs;
    if constexpr (KC > 0) {
      // rows of at most 256 * KC columns: read once, thread t holds columns t, t + 256, ...
      float v[KC];
      float s = 0.0f;
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        const int64_t j = k * 256 + threadIdx.x;
        v[k] = j < M ? Store<T>::load1(xr + j) : 0.0f;
        s += v[k];
      }
      mu = block_sum_256(s, lds) / m_f;
      float q = 0.0f;
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        const int64_t j = k * 256 + threadIdx.x;
        const float d = v[k] - mu;
        v[k] = d;
        q += j < M ? d * d : 0.0f;
      }
      const float var = block_sum_256(q, lds) / m_f;
      rs = 1.0f / sqrtf(var + eps);
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        const int64_t j = k * 256 + threadIdx.x;
        if (j < M) Store<T>::store1(yr + j, fmaf(v[k] * rs, gamma[j], beta[j]));
      }
    } else {
      float s = 0.0f;
      for (int64_t j = threadIdx.x; j < M; j += 256) s += Store<T>::load1(xr + j);
      mu = block_sum_256(s, lds) / m_f;
      float q = 0.0f;
      for (int64_t j = threadIdx.x; j < M; j += 256) {
        const float d = Store<T>::load1(xr + j) - mu;
        q += d * d;
      }
      const float var = block_sum_256(q, lds) / m_f;
      rs = 1.0f / sqrtf(var + eps);
      for (int64_t j = threadIdx.x; j < M; j += 256) {
        const float d = Store<T>::load1(xr + j) - mu;
        Store<T>::store1(yr + j, fmaf(d * rs, gamma[j], beta[j]));
      }
    }
    if (threadIdx.x == 0) {
      rstd_out[row] = rs;
      if (mean_out) mean_out[row] = mu;
    }
  }
}

// A "batch" is kGroups*R consecutive rows: lane group g takes rows base + r*kGroups + g, r < R.
// All R rows of a group are fetched (kept packed) before any arithmetic, so a group waits
// for memory once per batch.  LOOP = false: one batch per workgroup (grid = batches).
// LOOP = true: workgroups walk the batches grid-stride and fetch the next batch before they
// compute on the current one; the column sums stay in registers across batches, so the LDS
// tree and the partial store are paid once per workgroup however many rows it walks.
template <typename T, int LANES, int CH, int R, bool LOOP>
__global__ __launch_bounds__(kBwdThreads) void ln_bwd_kernel(
    const T* dy, const T* __restrict__ y, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ rstd, T* dx,
    float* __restrict__ partial, int64_t N, int M) {
  extern __shared__ float lds[];  // bwd_lds_bytes(): the tree's [slots][2][M] floats, >= 3*M
  constexpr int kGroups = kBwdThreads / LANES;
  constexpr int V = Store<T>::kVec;
  const int g = threadIdx.x / LANES;
  const int t = threadIdx.x % LANES;
  const int wave = threadIdx.x / kWave;
  const int lane = threadIdx.x & (kWave - 1);
  const int chunks = M / V;
  const float inv_m = 1.0f / static_cast<float>(M);
  const int64_t batch_rows = kGroups * R;
  __shared__ float2 red[2][kBwdWaves];
  static_assert(LANES <= kWave || R == 1, "rows over several waves: one row per group");
  int flip = 0;
  // gamma, 1/gamma and beta/gamma of the lane's columns live in its registers when that share
  // is at most 24 columns; otherwise in LDS (the first 3*M floats; the
  // same memory is reused by the reduction tree at the end), where every row re-reads the three
  // vectors twice: at 8 waves per compute unit that is microseconds of LDS time per batch.
  // The column sums are always in registers.
  constexpr bool kRegParams = CH * V <= 24;
  float* p_ga = lds;
  float* p_rg = lds + M;
  float* p_bg = lds + 2 * M;
  float r_ga[kRegParams ? CH : 1][V], r_rg[kRegParams ? CH : 1][V], r_bg[kRegParams ? CH : 1][V];
  // xhat and dy*gamma of the batch stay in registers between the two passes when they fit (128
  // registers; a workgroup of 8 waves has 256 per lane however few it uses): the second pass
  // then neither unpacks nor recomputes them.  Same arithmetic either way.
  constexpr bool kKeep = kRegParams && R * CH * V <= 64 && R * CH * 8 * (LOOP ? 2 : 1) <= 64;
  float k_h[kKeep ? R : 1][kKeep ? CH : 1][V], k_q[kKeep ? R : 1][kKeep ? CH : 1][V];
  float acc_g[CH][V], acc_b[CH][V];
#pragma unroll
  for (int c = 0; c < CH; ++c) {
#pragma unroll
    for (int i = 0; i < V; ++i) acc_g[c][i] = acc_b[c][i] = 0.0f;
  }

  auto fetch = [&](int64_t base, Raw<T> (&fd)[R][CH], Raw<T> (&fy)[R][CH], float (&fs)[R]) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t row = base + r * kGroups + g;
      fs[r] = 0.0f;
      if (row < N) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const int ch = c * LANES + t;
          if (ch < chunks) {
            fd[r][c].load(dy + row * M + ch * V);
            fy[r][c].load(y + row * M + ch * V);
          }
        }
        fs[r] = rstd[row];
      }
    }
  };

  int64_t base = static_cast<int64_t>(blockIdx.x) * batch_rows;
  Raw<T> rd[R][CH], ry[R][CH];
  float rs[R];
  fetch(base, rd, ry, rs);
  // parameters after the first rows are on their way
  if constexpr (kRegParams) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int ch = c * LANES + t;
      float be[V];
      if (ch < chunks) {
        load_floats<V>(gamma + ch * V, r_ga[c]);
        load_floats<V>(beta + ch * V, be);
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i) {
          r_ga[c][i] = 1.0f;
          be[i] = 0.0f;
        }
      }
#pragma unroll
      for (int i = 0; i < V; ++i) {
        // reciprocal by the hardware estimate and one Newton step (within 1 ulp): a lane does this
        // for each of its columns in every workgroup, and the IEEE division costs four times as much
        const float est = __builtin_amdgcn_rcpf(r_ga[c][i]);
        r_rg[c][i] = fmaf(fmaf(-r_ga[c][i], est, 1.0f), est, est);
        r_bg[c][i] = be[i] * r_rg[c][i];
      }
    }
  } else {
    for (int j = threadIdx.x; j < M; j += kBwdThreads) {
      const float gj = gamma[j];
      const float rj = 1.0f / gj;
      p_ga[j] = gj;
      p_rg[j] = rj;
      p_bg[j] = beta[j] * rj;
    }
    lds_barrier();
  }
  while (base < N) {
    const int64_t next = base + static_cast<int64_t>(gridDim.x) * batch_rows;
    Raw<T> nd[R][CH], ny[R][CH];  // unused (and eliminated) without LOOP
    float ns[R];
    if constexpr (LOOP) {
      if (next < N) fetch(next, nd, ny, ns);
    }
    // pass 1: the two row sums of every row (and the column accumulators); the R butterfly
    // chains are independent, so their latencies overlap
    float c1[R], c2[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t row = base + r * kGroups + g;
      c1[r] = c2[r] = 0.0f;
      if (row >= N) continue;  // uniform over the lane group
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int ch = c * LANES + t;
        if (ch < chunks) {
          float d8[V], y8[V], ga[V], rg[V], bg[V];
          rd[r][c].unpack(d8);
          ry[r][c].unpack(y8);
          if constexpr (kRegParams) {
#pragma unroll
            for (int i = 0; i < V; ++i) {
              ga[i] = r_ga[c][i];
              rg[i] = r_rg[c][i];
              bg[i] = r_bg[c][i];
            }
          } else {
            load_floats<V>(p_ga + ch * V, ga);
            load_floats<V>(p_rg + ch * V, rg);
            load_floats<V>(p_bg + ch * V, bg);
          }
#pragma unroll
          for (int i = 0; i < V; ++i) {
            const float h = fmaf(y8[i], rg[i], -bg[i]);  // xhat = (y - beta) / gamma
            const float q = d8[i] * ga[i];
            c1[r] = fmaf(q, h, c1[r]);
            c2[r] += q;
            acc_g[c][i] = fmaf(d8[i], h, acc_g[c][i]);
            acc_b[c][i] += d8[i];
            if constexpr (kKeep) {
              k_h[r][c][i] = h;
              k_q[r][c][i] = q;
            }
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      row_sum2<LANES>(c1[r], c2[r], red[flip]);
      flip ^= 1;
      c1[r] *= inv_m;
      c2[r] *= inv_m;
    }
    // pass 2: dx, from the kept xhat and dy*gamma or recomputing them from the packed registers
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t row = base + r * kGroups + g;
      if (row >= N) continue;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int ch = c * LANES + t;
        if (ch < chunks) {
          float o[V];
          if constexpr (kKeep) {
#pragma unroll
            for (int i = 0; i < V; ++i)
              o[i] = rs[r] * (k_q[r][c][i] - fmaf(k_h[r][c][i], c1[r], c2[r]));
          } else {
            float d8[V], y8[V], ga[V], rg[V], bg[V];
            rd[r][c].unpack(d8);
            ry[r][c].unpack(y8);
            if constexpr (kRegParams) {
#pragma unroll
              for (int i = 0; i < V; ++i) {
                ga[i] = r_ga[c][i];
                rg[i] = r_rg[c][i];
                bg[i] = r_bg[c][i];
              }
            } else {
              load_floats<V>(p_ga + ch * V, ga);
              load_floats<V>(p_rg + ch * V, rg);
              load_floats<V>(p_bg + ch * V, bg);
            }
#pragma unroll
            for (int i = 0; i < V; ++i) {
              const float h = fmaf(y8[i], rg[i], -bg[i]);
              o[i] = rs[r] * (d8[i] * ga[i] - fmaf(h, c1[r], c2[r]));
            }
          }
          store_piece<T>(dx + row * M + ch * V, o);
        }
      }
    }
    if constexpr (!LOOP) {
      break;
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          rd[r][c] = nd[r][c];
          ry[r][c] = ny[r][c];
        }
        rs[r] = ns[r];
      }
      base = next;
    }
  }
  // Column sums of the workgroup -> its [2][M] slot of `partial`.  First over the lane groups
  // that share a wave (fixed butterfly), then over the waves through LDS.  When a row takes
  // W > 1 waves, wave w holds the columns of part w % W of the row; the W waves of one row, whose
  // columns are disjoint, share one [2][M] LDS slot, so there are S = kBwdWaves / W slots to add.
  // The association is the same on both routes, a binary tree that pairs slot s with s + S/2,
  // then s + S/4, ...:
  //  - all S slots fit kOneStepLdsBytes: every wave writes its sums, one barrier, and each lane
  //    of the workgroup adds one 16-byte piece of the S slots and stores it;
  //  - else the tree runs through S/2 slots, a barrier pair per level, and the waves of slot 0
  //    store the result.
  // This tail is on the critical path of the kernel (the tree and the slot's store were each
  // measured at about a microsecond of it); running it before the last batch's dx is stored
  // hides the store but puts a barrier between the waves' loads and stores, and was slower.
#pragma unroll
  for (int c = 0; c < CH; ++c) {
#pragma unroll
    for (int i = 0; i < V; ++i) {
#pragma unroll
      for (int m = LANES; m < kWave; m <<= 1) {
        acc_g[c][i] += __shfl_xor(acc_g[c][i], m, kWave);
        acc_b[c][i] += __shfl_xor(acc_b[c][i], m, kWave);
      }
    }
  }
  const bool owner = lane < LANES;  // one copy per wave
  constexpr int kRowWaves = LANES > kWave ? LANES / kWave : 1;
  constexpr int S = kBwdWaves / kRowWaves;
  float* out = partial + static_cast<size_t>(blockIdx.x) * 2 * M;
  if (static_cast<size_t>(S) * 2 * M * sizeof(float) <= kOneStepLdsBytes) {
    if constexpr (!kRegParams) lds_barrier();  // the parameters in LDS are no longer read
    if (owner) {
      float* slot = lds + static_cast<size_t>(wave / kRowWaves) * 2 * M;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int ch = c * LANES + t;
        if (ch < chunks) {
          store_floats<V>(slot + ch * V, acc_g[c]);
          store_floats<V>(slot + M + ch * V, acc_b[c]);
        }
      }
    }
    lds_barrier();
    for (int j = threadIdx.x * 4; j < 2 * M; j += kBwdThreads * 4) {
      float v[S][4];
#pragma unroll
      for (int k = 0; k < S; ++k) load_floats<4>(lds + static_cast<size_t>(k) * 2 * M + j, v[k]);
#pragma unroll
      for (int half = S / 2; half >= 1; half >>= 1) {
#pragma unroll
        for (int k = 0; k < half; ++k) {
#pragma unroll
          for (int i = 0; i < 4; ++i) v[k][i] += v[k + half][i];
        }
      }
      store_floats<4>(out + j, v[0]);
    }
    return;
  }
#pragma unroll
  for (int half = kBwdWaves / 2; half >= kRowWaves; half >>= 1) {
    lds_barrier();
    if (wave >= half && wave < 2 * half && owner) {
      float* slot = lds + static_cast<size_t>((wave - half) / kRowWaves) * 2 * M;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int ch = c * LANES + t;
        if (ch < chunks) {
          store_floats<V>(slot + ch * V, acc_g[c]);
          store_floats<V>(slot + M + ch * V, acc_b[c]);
        }
      }
    }
    lds_barrier();
    if (wave < half && owner) {
      const float* slot = lds + static_cast<size_t>(wave / kRowWaves) * 2 * M;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int ch = c * LANES + t;
        if (ch < chunks) {
          float a[V], b[V];
          load_floats<V>(slot + ch * V, a);
          load_floats<V>(slot + M + ch * V, b);
#pragma unroll
          for (int i = 0; i < V; ++i) {
            acc_g[c][i] += a[i];
            acc_b[c][i] += b[i];
          }
        }
      }
    }
  }
  if (wave < kRowWaves && owner) {
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int ch = c * LANES + t;
      if (ch < chunks) {
        store_floats<V>(out + ch * V, acc_g[c]);
        store_floats<V>(out + M + ch * V, acc_b[c]);
      }
    }
  }
}

// Any M: one workgroup per row for dx; per-workgroup column partials are accumulated by
// walking rows blockIdx.x, blockIdx.x + gridDim.x, ... with thread j owning columns j, j+256...
// KC > 0: rows of at most 256 * KC columns; the thread's column sums and the gamma and beta of
// its columns live in registers and the partial slot is written once at the end.  KC == 0: any
// length; the sums are kept in the partial slot itself (private to the workgroup).
template <typename T, int KC>
__global__ __launch_bounds__(256) void ln_bwd_generic_kernel(
    const T* dy, const T* __restrict__ y, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ rstd, T* dx,
    float* __restrict__ partial, int64_t N, int64_t M) {
  __shared__ float lds[4];
  const float inv_m = 1.0f / static_cast<float>(M);
  float* pg = partial + static_cast<size_t>(blockIdx.x) * 2 * M;
  float* pb = pg + M;
  if constexpr (KC > 0) {
    float ag[KC], ab[KC], ga[KC], be[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      const int64_t j = k * 256 + threadIdx.x;
      ag[k] = ab[k] = 0.0f;
      ga[k] = j < M ? gamma[j] : 1.0f;
      be[k] = j < M ? beta[j] : 0.0f;
    }
    for (int64_t row = blockIdx.x; row < N; row += gridDim.x) {
      const T* dyr = dy + row * M;
      const T* yr = y + row * M;
      T* dxr = dx + row * M;
      float c1 = 0.0f, c2 = 0.0f;
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        const int64_t j = k * 256 + threadIdx.x;
        if (j < M) {
          const float d = Store<T>::load1(dyr + j);
          const float h = (Store<T>::load1(yr + j) - be[k]) / ga[k];
          const float q = d * ga[k];
          c1 = fmaf(q, h, c1);
          c2 += q;
          ag[k] = fmaf(d, h, ag[k]);
          ab[k] += d;
        }
      }
      c1 = block_sum_256(c1, lds) * inv_m;
      c2 = block_sum_256(c2, lds) * inv_m;
      const float rs = rstd[row];
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        const int64_t j = k * 256 + threadIdx.x;
        if (j < M) {
          const float d = Store<T>::load1(dyr + j);
          const float h = (Store<T>::load1(yr + j) - be[k]) / ga[k];
          Store<T>::store1(dxr + j, rs * (d * ga[k] - fmaf(h, c1, c2)));
        }
      }
    }
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      const int64_t j = k * 256 + threadIdx.x;
      if (j < M) {
        pg[j] = ag[k];
        pb[j] = ab[k];
      }
    }
  } else {
    for (int64_t j = threadIdx.x; j < M; j += 256) {
      pg[j] = 0.0f;
      pb[j] = 0.0f;
    }
    for (int64_t row = blockIdx.x; row < N; row += gridDim.x) {
      const T* dyr = dy + row * M;
      const T* yr = y + row * M;
      T* dxr = dx + row * M;
      float c1 = 0.0f, c2 = 0.0f;
      for (int64_t j = threadIdx.x; j < M; j += 256) {
        const float d = Store<T>::load1(dyr + j);
        const float h = (Store<T>::load1(yr + j) - beta[j]) / gamma[j];
        const float q = d * gamma[j];
        c1 = fmaf(q, h, c1);
        c2 += q;
        pg[j] = fmaf(d, h, pg[j]);
        pb[j] += d;
      }
      c1 = block_sum_256(c1, lds) * inv_m;
      c2 = block_sum_256(c2, lds) * inv_m;
      const float rs = rstd[row];
      for (int64_t j = threadIdx.x; j < M; j += 256) {
        const float d = Store<T>::load1(dyr + j);
        const float h = (Store<T>::load1(yr + j) - beta[j]) / gamma[j];
        Store<T>::store1(dxr + j, rs * (d * gamma[j] - fmaf(h, c1, c2)));
      }
    }
  }
}

// dgamma[j] = sum_p partial[p][0][j], dbeta[j] = sum_p partial[p][1][j].  A workgroup of 1024
// lanes owns 32 adjacent columns of the [2][M] row; its 32 slices each add every 32nd
// partial (all loads of a lane are independent and issued together), then the slices are
// combined through LDS in a fixed order.
constexpr int kFinCols = 32;   // 128 contiguous bytes per partial row
constexpr int kFinSlices = 32;
__global__ __launch_bounds__(kFinCols* kFinSlices) void ln_bwd_finalize_kernel(
    const float* __restrict__ partial, float* __restrict__ dgamma, float* __restrict__ dbeta,
    int parts, int64_t M) {
  __shared__ float lds[kFinSlices][kFinCols + 1];
  const int col = threadIdx.x % kFinCols;
  const int slice = threadIdx.x / kFinCols;
  const int64_t j2 = static_cast<int64_t>(blockIdx.x) * kFinCols + col;  // index into [2][M]
  float s = 0.0f;
  if (j2 < 2 * M) {
    const float* p0 = partial + j2;
    int p = slice;
    for (; p + 7 * kFinSlices < parts; p += 8 * kFinSlices) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p0[static_cast<size_t>(p + u * kFinSlices) * 2 * M];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; p < parts; p += kFinSlices) s += p0[static_cast<size_t>(p) * 2 * M];
  }
  lds[slice][col] = s;
  lds_barrier();
  if (slice == 0 && j2 < 2 * M) {
    float tot = 0.0f;
#pragma unroll
    for (int k = 0; k < kFinSlices; ++k) tot += lds[k][col];
    if (j2 < M) dgamma[j2] = tot;
    else dbeta[j2 - M] = tot;
  }
}

// The same sums in the same order with 16-byte loads: 8 lanes x 4 floats cover the 32 columns,
// so a workgroup is 4 waves instead of 16 and a wave's load touches 8 slices.  Needs whole
// 16-byte pieces in every [2][M] slot: M even.
constexpr int kFinVecLanes = kFinCols / 4;
__global__ __launch_bounds__(kFinVecLanes* kFinSlices) void ln_bwd_finalize4_kernel(
    const float* __restrict__ partial, float* __restrict__ dgamma, float* __restrict__ dbeta,
    int parts, int64_t M) {
  __shared__ float lds[kFinSlices][kFinCols + 4];
  const int q = threadIdx.x % kFinVecLanes;
  const int slice = threadIdx.x / kFinVecLanes;
  const int64_t j2 = static_cast<int64_t>(blockIdx.x) * kFinCols + q * 4;  // index into [2][M]
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (j2 < 2 * M) {
    const float* p0 = partial + j2;
    int p = slice;
    for (; p + 7 * kFinSlices < parts; p += 8 * kFinSlices) {
      float v[8][4];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        load_floats<4>(p0 + static_cast<size_t>(p + u * kFinSlices) * 2 * M, v[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
#pragma unroll
        for (int i = 0; i < 4; ++i) s[i] += v[u][i];
      }
    }
    for (; p < parts; p += kFinSlices) {
      float v[4];
      load_floats<4>(p0 + static_cast<size_t>(p) * 2 * M, v);
#pragma unroll
      for (int i = 0; i < 4; ++i) s[i] += v[i];
    }
  }
  store_floats<4>(&lds[slice][q * 4], s);
  lds_barrier();
  const int col = threadIdx.x;
  const int64_t j = static_cast<int64_t>(blockIdx.x) * kFinCols + col;
  if (col < kFinCols && j < 2 * M) {
    float tot = 0.0f;
#pragma unroll
    for (int k = 0; k < kFinSlices; ++k) tot += lds[k][col];
    if (j < M) dgamma[j] = tot;
    else dbeta[j - M] = tot;
  }
}

struct Shape {
  int lanes;
  int ch;
};

// Lanes per row and pieces per lane for a row of `pieces` 16-byte pieces: least padding, then
// the widest group.  ch == 0: no register-resident shape fits.  full_wave (the backward): a
// whole wave per row counts as unpadded while at most a third of its lanes' pieces are
// padding; one row per wave lets a lane group fetch up to 4 rows at once, which there is
// worth more than the idle lanes (measured at 384 and 768 columns; the forward loses by it).
Shape pick_shape(int pieces, bool full_wave) {
  static const int wide[] = {1, 2, 3, 4, 6, 8, 12, 16};  // 64 lanes
  static const int narrow[] = {1, 2, 3};                 // 32 and 16 lanes
  Shape best = {0, 0};
  int best_waste = 1 << 30;
  for (int lanes = 64; lanes >= 16; lanes >>= 1) {
    const int need = (pieces + lanes - 1) / lanes;
    const int* allowed = lanes == 64 ? wide : narrow;
    const int count = lanes == 64 ? 8 : 3;
    for (int k = 0; k < count; ++k) {
      if (allowed[k] >= need) {
        int waste = lanes * allowed[k] - pieces;
        if (full_wave && lanes == 64 && waste * 3 <= lanes * allowed[k]) waste = 0;
        if (waste < best_waste) {
          best_waste = waste;
          best = {lanes, allowed[k]};
        }
        break;
      }
    }
  }
  return best;
}

// A row whose pieces per lane on one wave would exceed max_ch is spread over 2 or 4 waves (at
// most 4 pieces per lane there).
Shape widen_shape(Shape one, int pieces, int max_ch, int max_lanes) {
  if (one.ch == 0 || (one.lanes == kWave && one.ch > max_ch)) {  // no one-wave shape, or too many pieces
    for (int lanes = 2 * kWave; lanes <= max_lanes; lanes *= 2) {
      const int need = (pieces + lanes - 1) / lanes;
      if (need <= max_ch || lanes == max_lanes) {
        if (need <= 4) return {lanes, need};
        if (lanes == max_lanes && need <= 8) return {lanes, need <= 6 ? 6 : 8};
        break;
      }
    }
  }
  return one;
}

}  // namespace

#define TEMPO_LN_DISPATCH(LAUNCH)                                                          \
  switch (sh.lanes * 100 + sh.ch) {                                                        \
    case 6401: LAUNCH(64, 1); break;                                                       \
    case 6402: LAUNCH(64, 2); break;                                                       \
    case 6403: LAUNCH(64, 3); break;                                                       \
    case 6404: LAUNCH(64, 4); break;                                                       \
    case 6406: LAUNCH(64, 6); break;                                                       \
    case 6408: LAUNCH(64, 8); break;                                                       \
    case 6412: LAUNCH(64, 12); break;                                                      \
    case 6416: LAUNCH(64, 16); break;                                                      \
    case 3201: LAUNCH(32, 1); break;                                                       \
    case 3202: LAUNCH(32, 2); break;                                                       \
    case 3203: LAUNCH(32, 3); break;                                                       \
    case 1601: LAUNCH(16, 1); break;                                                       \
    case 1602: LAUNCH(16, 2); break;                                                       \
    case 1603: LAUNCH(16, 3); break;                                                       \
    case 12801: LAUNCH(128, 1); break;                                                     \
    case 12802: LAUNCH(128, 2); break;                                                     \
    case 12803: LAUNCH(128, 3); break;                                                     \
    case 12804: LAUNCH(128, 4); break;                                                     \
    case 25601: LAUNCH(256, 1); break;                                                     \
    case 25602: LAUNCH(256, 2); break;                                                     \
    case 25603: LAUNCH(256, 3); break;                                                     \
    case 25604: LAUNCH(256, 4); break;                                                     \
    case 25606: LAUNCH(256, 6); break;                                                     \
    case 25608: LAUNCH(256, 8); break;                                                     \
    case 51202: LAUNCH(512, 2); break;                                                     \
    case 51204: LAUNCH(512, 4); break;                                                     \
    default: return TEMPO_ERR_UNSUPPORTED;                                                 \
  }

// Rows per lane group that exist as kernels for a shape (keeps the number of instantiations
// down): 4 only for one or two pieces per lane on full-wave groups, 2 up to four pieces.
template <int L, int C>
constexpr int max_rows() {
  return L > 64 ? 1 : ((C <= 2 && L == 64) ? 4 : (C <= 4 ? 2 : 1));
}

template <typename T, int L, int C>
static void ln_fwd_go(int rr, bool loop, int grid, hipStream_t st, const void* x, const float* gamma,
                      const float* beta, void* y, float* rstd, float* mean, int64_t N, int64_t M,
                      float eps) {
  if constexpr ((std::is_same<T, bf16_t>::value && C > 4 && L > kWave) || L > kFwdThreads) {
    // shapes that exist for float32 only, or for the backward only (fast_shape never picks them here)
  } else {
    auto go = [&](auto rows, auto lp) {
      hipLaunchKernelGGL((ln_fwd_kernel<T, L, C, decltype(rows)::value, decltype(lp)::value>),
                         dim3(grid), dim3(kFwdThreads), 0, st, static_cast<const T*>(x), gamma, beta,
                         static_cast<T*>(y), rstd, mean, N, static_cast<int>(M), eps);
    };
    using std::integral_constant;
    if constexpr (C == 1 && L <= 64) {
      if (rr == 4) {
        if (loop) return go(integral_constant<int, 4>{}, std::true_type{});
        return go(integral_constant<int, 4>{}, std::false_type{});
      }
    }
    if constexpr (C <= 2 && L <= 64) {
      if (rr == 2) {
        if (loop) return go(integral_constant<int, 2>{}, std::true_type{});
        return go(integral_constant<int, 2>{}, std::false_type{});
      }
    }
    if (loop) return go(integral_constant<int, 1>{}, std::true_type{});
    go(integral_constant<int, 1>{}, std::false_type{});
  }
}

static bool fast_shape(int64_t M, tempo_dtype dt, bool backward, Shape* sh) {
  const int vec = dt == TEMPO_F32 ? 4 : 8;
  if (M % vec != 0 || M / vec > (dt == TEMPO_F32 ? kMaxFastPiecesF32 : kMaxFastPieces)) return false;
  const int pieces = static_cast<int>(M / vec);
  *sh = widen_shape(pick_shape(pieces, backward), pieces,
                    tune_get(backward ? kTuneLnBwdMaxPieces : kTuneLnFwdMaxPieces), 256);
  // Backward: four waves whose lanes would own more than 24 columns each (parameters in LDS,
  // read twice per element) give the row to all eight waves, which halves the columns per lane
  // and keeps the parameters in registers.
  if (backward && sh->lanes == 256 && sh->ch * vec > 24) *sh = {kBwdThreads, sh->ch / 2};
  return sh->ch != 0;
}

tempo_status launch_layernorm_fwd(const void* x, const float* gamma, const float* beta, void* y,
                                  float* rstd, float* mean, int64_t N, int64_t M, float eps,
                                  tempo_dtype dt, hipStream_t st) {
  Shape sh;
  int64_t cap = static_cast<int64_t>(compute_units()) * tune_get(kTuneLnFwdBlocksPerCu);
  if (fast_shape(M, dt, false, &sh)) {
    // rows per lane group, if the knob allows more than one: 4 for rows of one piece per lane, 2
    // for two pieces, so that a lane has 4 pieces in flight (and as many fetched ahead when the
    // workgroups loop); rows of one piece also take one more workgroup per compute unit.
    // Measured on 16384 x 512 and 65536 x 256 bf16: 9-10 % faster than 2 rows.
    const int tuned = tune_get(kTuneLnFwdRows);
    int rr = (sh.ch <= 2 && sh.lanes <= kWave && tuned >= 2) ? (sh.ch == 1 ? 4 : 2) : 1;
    if (rr == 4) cap += compute_units();
    int groups = (kFwdThreads / sh.lanes) * rr;
    int64_t want = (N + groups - 1) / groups;
    // Rows of two pieces whose workgroups would walk five batches of two rows or more: one row
    // at a time and one more workgroup per compute unit instead (32768 and 65536 rows of 1024
    // bf16 columns: 5-6 % faster; up to 16384 rows the two-row form is as fast or faster).
    if (rr == 2 && want >= 5 * cap) {
      rr = 1;
      cap += compute_units();
      groups = kFwdThreads / sh.lanes;
      want = (N + groups - 1) / groups;
    }
    const bool loop = want > cap;
    const int grid = static_cast<int>(loop ? cap : want);
#define TEMPO_LAUNCH(L, C)                                                                   \
  do {                                                                                       \
    if (dt == TEMPO_F32) ln_fwd_go<float, L, C>(rr, loop, grid, st, x, gamma, beta, y, rstd, mean, N, M, eps);   \
    else ln_fwd_go<bf16_t, L, C>(rr, loop, grid, st, x, gamma, beta, y, rstd, mean, N, M, eps);    \
  } while (0)
    TEMPO_LN_DISPATCH(TEMPO_LAUNCH)
#undef TEMPO_LAUNCH
  } else {
    // one row per workgroup at a time: as many workgroups as a compute unit holds (8 of 256 lanes)
    const int64_t most = static_cast<int64_t>(compute_units()) * 8;
    const int grid = static_cast<int>(N < most ? N : most);
    auto go = [&](auto tag, auto kc) {
      using T = decltype(tag);
      hipLaunchKernelGGL((ln_fwd_generic_kernel<T, decltype(kc)::value>), dim3(grid), dim3(256), 0,
                         st, static_cast<const T*>(x), gamma, beta, static_cast<T*>(y), rstd, mean, N,
                         M, eps);
    };
    auto by_length = [&](auto tag) {  // columns per thread held in registers: 8, 20, or none
      if (M <= 256 * 8) go(tag, std::integral_constant<int, 8>{});
      else if (M <= 256 * 20) go(tag, std::integral_constant<int, 20>{});
      else go(tag, std::integral_constant<int, 0>{});
    };
    if (dt == TEMPO_F32) by_length(float{});
    else by_length(bf16_t{});
  }
  return launch_status();
}

// Launch plan of the register-resident backward kernel.  Rows per lane group and batch (r):
// as many as the knob allows while the packed rows stay within ~64 registers and the grid
// keeps one workgroup per compute unit.  If that leaves more batches than the knob's number of
// workgroups per compute unit (default 1), workgroups loop with prefetch instead (two batches
// are then held in registers: half the rows per batch for one-piece rows, one row otherwise) on
// a grid of that many workgroups per compute unit.  A grid that does not loop has exactly one
// workgroup per batch, however many that is.
struct BwdPlan {
  int r;
  bool loop;
  int grid;
};
static BwdPlan bwd_plan(int64_t N, const Shape& sh) {
  const int tuned = tune_get(kTuneLnBwdRowsPerGroup);
  const int regs_per_row = sh.ch * 8;  // dy and y, 4 registers per packed piece
  const int64_t groups = kBwdThreads / sh.lanes;
  const int cus = compute_units();
  auto batches = [&](int r) { return (N + groups * r - 1) / (groups * r); };
  int r = tuned >= 4 ? 4 : (tuned >= 2 ? 2 : 1);
  const int avail =  // max_rows<L, C>()
      sh.lanes > 64 ? 1 : ((sh.ch <= 2 && sh.lanes == 64) ? 4 : (sh.ch <= 4 ? 2 : 1));
  if (r > avail) r = avail;
  while (r > 1 && (r * regs_per_row > 64 || batches(r) < cus)) r >>= 1;
  const int64_t most = static_cast<int64_t>(tune_get(kTuneLnBwdLoopBlocksPerCu)) * cus;
  BwdPlan p;
  if (batches(r) > most) {
    p.loop = true;
    p.r = (r > 1 && sh.ch == 1) ? r / 2 : 1;  // measured: rows of 2 pieces per lane loop best alone
    p.grid = static_cast<int>(most);
  } else {
    p.loop = false;
    p.r = r;
    p.grid = static_cast<int>(batches(r));  // <= most <= 65536 * compute units
  }
  if (p.grid < 1) p.grid = 1;
  return p;
}

// Dynamic LDS of the backward kernel: the column sums' slots (one per kRowWaves waves: all of
// them when they fit kOneStepLdsBytes, else those of the upper half of the workgroup for the
// tree), or the three parameter vectors when they live in LDS.
static size_t bwd_lds_bytes(const Shape& sh, int64_t M, tempo_dtype dt) {
  const int row_waves = sh.lanes > kWave ? sh.lanes / kWave : 1;
  const int all = kBwdWaves / row_waves;
  const size_t one_step = static_cast<size_t>(all) * 2 * M * sizeof(float);
  const int slots = one_step <= kOneStepLdsBytes ? all : (all / 2 > 0 ? all / 2 : 1);
  const int vec = dt == TEMPO_F32 ? 4 : 8;
  const bool reg_params = sh.ch * vec <= 24;  // kRegParams of ln_bwd_kernel
  size_t floats = static_cast<size_t>(slots) * 2 * M;
  if (!reg_params && floats < static_cast<size_t>(3) * M) floats = static_cast<size_t>(3) * M;
  return floats * sizeof(float);
}

// Launches the register-resident backward kernel; returns the number of workgroups used (the
// number of partial slots written).  A looping launch is trimmed to the workgroups that are
// resident at once, so that no second round of workgroups repeats the reduction epilogue.
template <typename T, int L, int C>
static int ln_bwd_go(const BwdPlan& plan, size_t lds_bytes, hipStream_t st, const void* dy,
                     const void* y, const float* gamma, const float* beta, const float* rstd,
                     void* dx, float* workspace, int64_t N, int64_t M) {
  int grid = plan.grid;
  if constexpr ((std::is_same<T, bf16_t>::value && C > 4 && L > kWave) ||
                (L == kBwdThreads && C != (std::is_same<T, bf16_t>::value ? 2 : 4))) {
    return grid;  // shapes that exist for the other dtype only
  } else {
    auto go = [&](auto rows, auto loop) {
      auto kernel = ln_bwd_kernel<T, L, C, decltype(rows)::value, decltype(loop)::value>;
      if (decltype(loop)::value) {
        static std::atomic<int> resident{0};  // workgroups per compute unit, per instantiation
        int per_cu = resident.load(std::memory_order_relaxed);
        if (per_cu == 0) {
          if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kBwdThreads,
                                                           lds_bytes) != hipSuccess || per_cu < 1) {
            (void)hipGetLastError();
            per_cu = 1;
          }
          resident.store(per_cu, std::memory_order_relaxed);
        }
        const int fit = per_cu * compute_units();
        if (grid > fit) grid = fit;
      }
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(kBwdThreads), lds_bytes, st,
                         static_cast<const T*>(dy), static_cast<const T*>(y), gamma, beta, rstd,
                         static_cast<T*>(dx), workspace, N, static_cast<int>(M));
    };
    using std::integral_constant;
    if (plan.loop) {
      if constexpr (max_rows<L, C>() >= 4) {  // looping holds two batches: half the rows
        if (plan.r == 2) {
          go(integral_constant<int, 2>{}, std::true_type{});
          return grid;
        }
      }
      go(integral_constant<int, 1>{}, std::true_type{});
      return grid;
    }
    if constexpr (max_rows<L, C>() >= 4) {
      if (plan.r == 4) {
        go(integral_constant<int, 4>{}, std::false_type{});
        return grid;
      }
    }
    if constexpr (max_rows<L, C>() >= 2) {
      if (plan.r >= 2) {
        go(integral_constant<int, 2>{}, std::false_type{});
        return grid;
      }
    }
    go(integral_constant<int, 1>{}, std::false_type{});
    return grid;
  }
}

// Everything a backward launch depends on, taken from the knobs once: the workspace check and
// the launch of one call always see the same plan.
struct BwdLaunch {
  bool fast;    // register-resident kernel (else the any-M kernel)
  Shape sh;
  BwdPlan plan;
  int slots;    // partial [2][M] slots the row kernel may write: an upper bound of its grid
};
static BwdLaunch bwd_launch(int64_t N, int64_t M, tempo_dtype dt) {
  BwdLaunch b;
  b.fast = fast_shape(M, dt, true, &b.sh);
  if (b.fast) {
    b.plan = bwd_plan(N, b.sh);
    b.slots = b.plan.grid;
  } else {
    // one row per workgroup, strided; four 256-lane workgroups per compute unit, and a workspace
    // of at most 1024 slots
    b.plan = {1, true, static_cast<int>(N > 1024 ? 1024 : (N < 1 ? 1 : N))};
    b.slots = b.plan.grid;
  }
  return b;
}
static size_t slot_bytes(const BwdLaunch& b, int64_t M) {
  return static_cast<size_t>(b.slots) * 2 * static_cast<size_t>(M) * sizeof(float);
}

size_t layernorm_bwd_workspace_bytes(int64_t N, int64_t M, tempo_dtype dt) {
  return slot_bytes(bwd_launch(N, M, dt), M);
}

tempo_status launch_layernorm_bwd(const void* dy, const void* y, const float* gamma,
                                  const float* beta, const float* rstd, void* dx, float* dgamma,
                                  float* dbeta, float* workspace, size_t workspace_bytes,
                                  int64_t N, int64_t M, tempo_dtype dt, hipStream_t st) {
  const BwdLaunch b = bwd_launch(N, M, dt);
  if (workspace_bytes < slot_bytes(b, M)) return TEMPO_ERR_WORKSPACE;
  int grid = b.plan.grid;
  if (b.fast) {
    const Shape sh = b.sh;
    const size_t lds_bytes = bwd_lds_bytes(sh, M, dt);
    const BwdPlan plan = b.plan;
#define TEMPO_LAUNCH(L, C)                                                                   \
  do {                                                                                       \
    if (dt == TEMPO_F32) grid = ln_bwd_go<float, L, C>(plan, lds_bytes, st, dy, y, gamma, beta, rstd, dx, workspace, N, M);   \
    else grid = ln_bwd_go<bf16_t, L, C>(plan, lds_bytes, st, dy, y, gamma, beta, rstd, dx, workspace, N, M);                  \
  } while (0)
    TEMPO_LN_DISPATCH(TEMPO_LAUNCH)
#undef TEMPO_LAUNCH
  } else {
    auto go = [&](auto tag, auto kc) {
      using T = decltype(tag);
      hipLaunchKernelGGL((ln_bwd_generic_kernel<T, decltype(kc)::value>), dim3(grid), dim3(256), 0,
                         st, static_cast<const T*>(dy), static_cast<const T*>(y), gamma, beta, rstd,
                         static_cast<T*>(dx), workspace, N, M);
    };
    auto by_length = [&](auto tag) {  // columns per thread held in registers: 8, 20, or none
      if (M <= 256 * 8) go(tag, std::integral_constant<int, 8>{});
      else if (M <= 256 * 20) go(tag, std::integral_constant<int, 20>{});
      else go(tag, std::integral_constant<int, 0>{});
    };
    if (dt == TEMPO_F32) by_length(float{});
    else by_length(bf16_t{});
  }
  if (hipGetLastError() != hipSuccess) return TEMPO_ERR_LAUNCH;
  const int fgrid = static_cast<int>((2 * M + kFinCols - 1) / kFinCols);
  if (M % 2 == 0)
    hipLaunchKernelGGL(ln_bwd_finalize4_kernel, dim3(fgrid), dim3(kFinVecLanes * kFinSlices), 0, st,
                       workspace, dgamma, dbeta, grid, M);
  else
    hipLaunchKernelGGL(ln_bwd_finalize_kernel, dim3(fgrid), dim3(kFinCols * kFinSlices), 0, st,
                       workspace, dgamma, dbeta, grid, M);
  return launch_status();
}

// Scratch for callers that cannot allocate: one array per GPU, living in the code object.  Its
// name is only a host-side handle; the address kernels can use is looked up once per device.
static __device__ __align__(256) unsigned char scratch[TEMPO_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

tempo_status static_scratch(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return TEMPO_ERR_LAUNCH;
  }
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {  // first call on this device (threads racing here find the same address)
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return TEMPO_ERR_LAUNCH;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return TEMPO_OK;
}

}  // namespace tempo
