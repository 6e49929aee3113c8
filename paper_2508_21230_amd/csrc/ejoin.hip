// Brute-force Euclidean-distance epsilon self-join for gfx950 (MI355X): kernels and C ABI.
//
// Method (arXiv 2508.21230, Section 3.1): Step 1 norms s_i, Step 2 Gram products a_ij on the
// matrix cores with FP16 inputs / FP32 accumulation, Step 3 dist^2 = s_i + s_j - 2 a_ij, then
// the "<= epsilon" filter of Section 2.2.1.  The tiling below is designed for CDNA4 (64-wide
// wavefronts, v_mfma_f32_32x32x16_f16, 160 KB LDS with 64 banks, 8 XCDs with private L2s); the
// paper's A100 tiling (Section 3.2-3.3) is prior art, not the blueprint.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include <math.h>
#include <new>

#include "ejoin.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));

#define EJ_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define EJ_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

// ------------------------------------------------------------------------------------------
// Tiling constants
// ------------------------------------------------------------------------------------------
constexpr int TILE = 256;          // a workgroup computes a TILE x TILE block of the distance matrix
constexpr int KSLICE = 64;         // coordinates per LDS stage (128 B per row)
constexpr int THREADS = 512;       // 8 wavefronts: 2 (rows) x 4 (columns), wave tile 128 x 64
constexpr int SB = 16;             // tiles per super-block edge (one super-block = 256 tiles = one pass of the chip)
constexpr int PANEL_BYTES = TILE * KSLICE * 2;      // 32 KB : one operand panel of one stage
constexpr int STAGE_BYTES = 2 * PANEL_BYTES;        // A panel + B panel
constexpr int NORM_OFF = 2 * STAGE_BYTES;           // two stages, then the norm staging area
constexpr int NORM_BYTES = 2 * 2 * TILE * 4;        // [tile parity][A|B][TILE] floats
constexpr int SLOT_OFF = NORM_OFF + NORM_BYTES;     // [tile parity] next-tile slots (int4 each)
constexpr int LDS_BYTES = SLOT_OFF + 2 * 16;
constexpr int NUM_XCD = 8;

// LDS layout of a panel: row r (0..255) occupies bytes [r*128, r*128+128); its eight 16-byte
// chunks are stored permuted, chunk c at position c ^ ((r >> 1) & 7).  With 64 banks of 4 B a
// ds_read_b128 serves 16 lanes per clock; 16 consecutive rows at the same logical chunk then
// fall into 16 distinct 16-byte bank groups (measured: 241 B/clk/CU against 128 for r & 7).
// This is the role the XOR swizzle of Section 3.3.5 (Eq. 2) plays on the A100's 32 banks.
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

struct JoinArgs {
  const uint16_t* X;
  const float* s;
  int64_t n;
  int64_t ld;
  int nslices;  // roundup(d, 64) / 64
  float eps2;
  uint32_t ntiles;  // ceil(n / TILE)
  uint32_t nsb;     // ceil(ntiles / SB)
  uint32_t items_per_xcd;
  uint32_t* queue;  // NUM_XCD work counters
  // pair mode
  uint32_t* pairs;
  float* dist2;
  unsigned long long capacity;
  unsigned long long* n_pairs;
  // count mode
  uint32_t* counts;
  unsigned long long* total;
};

// ------------------------------------------------------------------------------------------
// Small kernels
// ------------------------------------------------------------------------------------------
__global__ void k_reset(uint32_t* queue, unsigned long long* c0, unsigned long long* c1) {
  if (threadIdx.x < NUM_XCD) queue[threadIdx.x] = 0;
  if (threadIdx.x == 0) {
    if (c0) *c0 = 0;
    if (c1) *c1 = 0;
  }
}

__global__ void k_fill_u32(uint32_t* p, int64_t n, uint32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Step 1 (Section 3.1): s_i = sum_k x_ik^2.  One wavefront per 32 consecutive points; the 32 x 32
// Gram block of those points is accumulated with the same MFMA steps, in the same k order, as
// the join kernel uses, and its diagonal is stored.  That makes s_i bit-identical to a_ii, and
// to a_ij for a duplicate j of i, so duplicates come out at distance exactly 0.  (The paper
// matches its norm rounding to its tensor cores' for the same reason.)
__global__ __launch_bounds__(256) void k_norms(const uint16_t* __restrict__ X, int64_t n, int64_t ld, int k16steps,
                                               float* __restrict__ s) {
  const int lane = threadIdx.x & 63;
  const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t row0 = blk * 32;
  if (row0 >= n) return;
  int64_t row = row0 + (lane & 31);
  if (row >= n) row = n - 1;
  const half8* p = reinterpret_cast<const half8*>(X + row * ld) + (lane >> 5);
  float16v acc;
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int k = 0; k < k16steps; ++k) {
    half8 a = p[2 * k];
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, a, acc, 0, 0, 0);
  }
  // element (row, col) of the 32x32 block sits in lane (col + 32*hi), register r with
  // row = 8*(r/4) + 4*hi + r%4 ; the diagonal element of column c is in the lane whose
  // hi equals bit 2 of c, register 4*(c/8) + c%4.
  const int c = lane & 31, hi = lane >> 5;
  if (((c >> 2) & 1) == hi && row0 + c < n) {
    const int want = 4 * (c >> 3) + (c & 3);
    float v = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (r == want) v = acc[r];
    s[row0 + c] = v;
  }
}

// Dense block of squared distances with the join's arithmetic: one wavefront per 32 x 32 block.
__global__ __launch_bounds__(64) void k_dist2_tile(const uint16_t* __restrict__ X, const float* __restrict__ s, int64_t n,
                                                  int64_t ld, int k16steps, int64_t i0, int64_t j0, int rows, int cols,
                                                  float* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int bi = blockIdx.y * 32, bj = blockIdx.x * 32;
  int64_t ra = i0 + bi + (lane & 31), rb = j0 + bj + (lane & 31);
  if (ra >= n) ra = n - 1;
  if (rb >= n) rb = n - 1;
  const half8* pa = reinterpret_cast<const half8*>(X + ra * ld) + (lane >> 5);
  const half8* pb = reinterpret_cast<const half8*>(X + rb * ld) + (lane >> 5);
  float16v acc;
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int k = 0; k < k16steps; ++k) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(pa[2 * k], pb[2 * k], acc, 0, 0, 0);
  const int c = bj + (lane & 31), hi = lane >> 5;
  if (c < cols) {
    const float sj = s[j0 + c];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rr = bi + 8 * (r >> 2) + 4 * hi + (r & 3);
      if (rr < rows) {
        const float t = s[i0 + rr] + sj;
        out[(int64_t)rr * cols + c] = fmaxf(fmaf(-2.f, acc[r], t), 0.f);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// The join kernel
// ------------------------------------------------------------------------------------------
// Work distribution (the counterpart of the paper's work queue that orders block tiles in small
// squares for L2 reuse, Section 3.3.1, re-derived for 8 XCDs with private 4 MB L2s):
//   * the upper triangle of the tile grid is cut into super-blocks of 16 x 16 tiles, enumerated
//     row-major; one super-block is one pass of the 256 CUs, so at any time the chip works on
//     (16+16) x 256 rows of X, which the memory-side cache holds;
//   * inside a super-block each XCD owns an 8 x 4 rectangle of tiles (12 row panels shared by its
//     32 CUs through its own L2); the rectangle rotates with the super-block index so that
//     partially empty (diagonal, ragged) super-blocks do not starve the same XCD every time;
//   * workgroup w runs on XCD w % 8 (hardware round-robin, verified on device) and pops tiles of
//     its XCD from a per-XCD counter, so imbalance inside an XCD is absorbed dynamically.
// item t of XCD x  ->  tile (I, J) or "nothing here" (below the diagonal / outside the grid).
__device__ __forceinline__ bool decode_item(const JoinArgs& a, uint32_t xcd, uint32_t t, uint32_t& I, uint32_t& J) {
  const uint32_t sbi = t >> 5, slot = t & 31;
  const uint32_t nsb = a.nsb;
  // row-major upper triangle: row P starts at P*nsb - P(P-1)/2
  const double b = 2.0 * nsb + 1.0;
  uint32_t P = (uint32_t)((b - sqrt(b * b - 8.0 * (double)sbi)) * 0.5);
  if (P >= nsb) P = nsb - 1;
  auto start = [nsb](uint32_t p) { return (uint64_t)p * nsb - ((uint64_t)p * (p - 1)) / 2; };
  while (P > 0 && start(P) > sbi) --P;
  while (P + 1 < nsb && start(P + 1) <= sbi) ++P;
  const uint32_t Q = P + (uint32_t)(sbi - start(P));
  const uint32_t xp = (xcd + sbi) & 7;
  I = P * SB + (xp >> 2) * 8 + (slot >> 2);
  J = Q * SB + (xp & 3) * 4 + (slot & 3);
  return I <= J && J < a.ntiles;
}

template <bool COUNT>
__global__ __launch_bounds__(THREADS) void k_join(const JoinArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int r32 = lane & 31, hi = lane >> 5;
  const uint32_t xcd = blockIdx.x & (NUM_XCD - 1);
  int4* slots = reinterpret_cast<int4*>(lds + SLOT_OFF);

  // thread 0 pops items of this XCD.  `resolve` turns a raw item into {I, J, valid, 0}, popping
  // further items while they are empty (below the diagonal / outside the grid).
  auto resolve = [&](uint32_t t) -> int4 {
    for (;;) {
      if (t >= a.items_per_xcd) return make_int4(0, 0, 0, 0);
      uint32_t I, J;
      if (decode_item(a, xcd, t, I, J)) return make_int4((int)I, (int)J, 1, 0);
      t = atomicAdd(&a.queue[xcd], 1u);
    }
  };

  // --- global->LDS copy addressing: wave w copies rows 8*(w + 8q) .. +7 (q = 0..3) of both panels;
  // lane l handles row +l/8 and the LDS chunk position l%8, i.e. the logical chunk (l%8) ^ swz(row).
  const int drow = lane >> 3;
  const char* Xb = reinterpret_cast<const char*>(a.X);
  const int64_t rowbytes = a.ld * 2;
  const char* gA[4];
  const char* gB[4];
  auto set_tile_ptrs = [&](int I, int J) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int row = 8 * (wave + 8 * q) + drow;
      const int chunk = (lane & 7) ^ swz(row);
      int64_t ra = (int64_t)I * TILE + row, rb = (int64_t)J * TILE + row;
      if (ra >= a.n) ra = a.n - 1;  // rows past the end are clamped; their results are masked by s = +inf
      if (rb >= a.n) rb = a.n - 1;
      gA[q] = Xb + ra * rowbytes + chunk * 16;
      gB[q] = Xb + rb * rowbytes + chunk * 16;
    }
  };
  auto issue_slice = [&](int ks, int stage) {
    char* base = lds + stage * STAGE_BYTES;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      __builtin_amdgcn_global_load_lds(EJ_GLB(gA[q] + (int64_t)ks * (KSLICE * 2)), EJ_LDS(base + (wave + 8 * q) * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(EJ_GLB(gB[q] + (int64_t)ks * (KSLICE * 2)),
                                       EJ_LDS(base + PANEL_BYTES + (wave + 8 * q) * 1024), 16, 0, 0);
    }
  };
  // norm of this thread's row (threads 0..255: rows of the tile, A side; 256..511: columns, B side);
  // rows past the end get +inf, so none of their pairs can pass the filter
  auto load_norm = [&](int I, int J) -> float {
    const int64_t g = (tid < TILE) ? (int64_t)I * TILE + tid : (int64_t)J * TILE + (tid - TILE);
    return (g < a.n) ? a.s[g] : __builtin_inff();
  };
  auto norm_buf = [&](int parity) -> float* { return reinterpret_cast<float*>(lds + NORM_OFF) + parity * (2 * TILE); };

  // --- fragment read addressing (byte offsets inside a stage)
  // A operand of v_mfma_f32_32x32x16_f16: lane l supplies row l%32, coordinates 8*(l/32) .. +7 of the 16-wide step.
  int offA[4], offB[4];  // per 16-wide k step; m-tile / n-tile add 32 rows = 4096 B (swz unchanged: 32 % 16 == 0)
  {
    const int rowA = wm * 128 + r32, rowB = wn * 64 + r32;
#pragma unroll
    for (int k16 = 0; k16 < 4; ++k16) {
      offA[k16] = rowA * 128 + (((2 * k16 + hi) ^ swz(rowA)) << 4);
      offB[k16] = PANEL_BYTES + rowB * 128 + (((2 * k16 + hi) ^ swz(rowB)) << 4);
    }
  }

  float16v acc[4][2];

  // ---------------- prologue: first tile
  if (tid == 0) slots[0] = resolve(atomicAdd(&a.queue[xcd], 1u));
  __syncthreads();
  int4 cur = slots[0];
  uint32_t T = 0;  // tiles done by this workgroup
  uint32_t g = 0;  // k-slices done by this workgroup (stage = g & 1)
  if (cur.z) {
    norm_buf(0)[tid] = load_norm(cur.x, cur.y);
    set_tile_ptrs(cur.x, cur.y);
    issue_slice(0, 0);
  }
  uint32_t raw_next = 0;

  while (cur.z) {
    const int I = cur.x, J = cur.y;
    int4 nxt = make_int4(0, 0, 0, 0);
    float nxt_norm = 0.f;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;

    for (int ks = 0; ks < a.nslices; ++ks, ++g) {
      const bool last = (ks + 1 == a.nslices);
      // one-tile lookahead: thread 0 publishes the tile after this one before the barrier of
      // this tile's last slice (the raw item was popped a slice earlier, so its latency is hidden)
      if (last && tid == 0) {
        if (a.nslices == 1) raw_next = atomicAdd(&a.queue[xcd], 1u);
        slots[(T + 1) & 1] = resolve(raw_next);
      }
      // this wave's copies of slice ks have landed; after the barrier everybody's have, and
      // everybody is done reading the other stage (slice ks-1)
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (ks == 0 && a.nslices > 1 && tid == 0) raw_next = atomicAdd(&a.queue[xcd], 1u);
      if (!last) {
        issue_slice(ks + 1, (g + 1) & 1);
      } else {
        nxt = slots[(T + 1) & 1];
        if (nxt.z) {
          nxt_norm = load_norm(nxt.x, nxt.y);  // issued before the copies so that waiting for it does not wait for them
          set_tile_ptrs(nxt.x, nxt.y);
          issue_slice(0, (g + 1) & 1);
        }
      }
      const char* st = lds + (g & 1) * STAGE_BYTES;
#pragma unroll
      for (int k16 = 0; k16 < 4; ++k16) {
        half8 fa[4], fb[2];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) fa[mt] = *reinterpret_cast<const half8*>(st + offA[k16] + mt * 4096);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) fb[nt] = *reinterpret_cast<const half8*>(st + offB[k16] + nt * 4096);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[mt], fb[nt], acc[mt][nt], 0, 0, 0);
      }
    }
    // norms of the next tile go to the other parity's staging area; its last readers (epilogue of
    // tile T-1) are behind every wave that has passed this tile's first barrier
    if (nxt.z) norm_buf((T + 1) & 1)[tid] = nxt_norm;

    // ---------------- epilogue (Step 3 of Section 3.1 + the epsilon filter), fused
    // accumulator register r of tile (mt, nt) in lane l is the pair
    //   i = I*256 + wm*128 + mt*32 + 8*(r/4) + 4*(l/32) + r%4 ,  j = J*256 + wn*64 + nt*32 + l%32.
    {
      const float* nb = norm_buf(T & 1);
      const bool diag = (I == J);
      const uint32_t ibase = (uint32_t)I * TILE + wm * 128 + 4 * hi;
      const uint32_t jbase = (uint32_t)J * TILE + wn * 64 + r32;
      unsigned long long wave_hits = 0;
      // a wave tile of a diagonal block that lies entirely below the diagonal holds no pair i <= j
      const bool skip = diag && (wm * 128 >= wn * 64 + 64);
      if (!skip) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          const float sj = nb[TILE + wn * 64 + nt * 32 + r32];
          const uint32_t j = jbase + nt * 32;
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
              const float4v si4 = *reinterpret_cast<const float4v*>(nb + wm * 128 + mt * 32 + 8 * rq + 4 * hi);
#pragma unroll
              for (int rr = 0; rr < 4; ++rr) {
                const float d2 = fmaf(-2.f, acc[mt][nt][4 * rq + rr], si4[rr] + sj);
                const uint32_t i = ibase + mt * 32 + 8 * rq + rr;
                bool pass = d2 <= a.eps2;  // rows/columns past n carry s = +inf and never pass
                if (diag) pass = (i == j) ? (COUNT ? false : (i < a.n)) : (pass && i < j);
                const unsigned long long mask = __ballot(pass);
                if (mask) {
                  const uint32_t cnt = __popcll(mask);
                  if (COUNT) {
                    if (pass) {
                      atomicAdd(&a.counts[i], 1u);
                      atomicAdd(&a.counts[j], 1u);
                    }
                    wave_hits += cnt;
                  } else {
                    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                    unsigned long long base = 0;
                    if (rank == 0 && pass) base = atomicAdd(a.n_pairs, (unsigned long long)cnt);
                    // broadcast from the first passing lane
                    const int src = __ffsll((long long)mask) - 1;
                    const uint32_t blo = __builtin_amdgcn_readlane((uint32_t)base, src);
                    const uint32_t bhi = __builtin_amdgcn_readlane((uint32_t)(base >> 32), src);
                    base = ((unsigned long long)bhi << 32) | blo;
                    const unsigned long long idx = base + rank;
                    if (pass && idx < a.capacity) {
                      reinterpret_cast<uint2*>(a.pairs)[idx] = make_uint2(i, j);
                      if (a.dist2) a.dist2[idx] = (i == j) ? 0.f : fmaxf(d2, 0.f);
                    }
                  }
                }
              }
            }
          }
        }
      }
      if (COUNT && wave_hits && lane == 0) atomicAdd(a.total, wave_hits);
    }
    cur = nxt;
    ++T;
  }
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
}  // namespace

struct ejoin_ctx {
  int device;
  int num_cu;
  uint32_t* queue;              // NUM_XCD counters
  unsigned long long* scratch;  // 2 x u64 (unused outputs land here)
  float* s;                     // norms workspace
  int64_t s_cap;
  int profiling;
  hipEvent_t ev[4];
  int ev_valid;
  char hip_error[256];
};

namespace {

int fail_hip(ejoin_ctx* ctx, hipError_t e, const char* what) {
  if (ctx) snprintf(ctx->hip_error, sizeof(ctx->hip_error), "%s: %s", what, hipGetErrorString(e));
  (void)hipGetLastError();
  return EJOIN_EHIP;
}

#define EJ_TRY(call)                                     \
  do {                                                   \
    hipError_t e_ = (call);                              \
    if (e_ != hipSuccess) return fail_hip(ctx, e_, #call); \
  } while (0)

int check_common(const ejoin_ctx* ctx, const void* X, int64_t n, int32_t d, int64_t ld) {
  if (!ctx || !X) return EJOIN_EINVAL;
  if (n < 1 || n >= (int64_t)0xFFFFFFFFll - TILE) return EJOIN_EINVAL;
  if (d < 1 || d > 65536) return EJOIN_EINVAL;
  const int64_t dk = ((int64_t)d + KSLICE - 1) / KSLICE * KSLICE;
  if (ld < dk || (ld % KSLICE) != 0) return EJOIN_EINVAL;
  if ((reinterpret_cast<uintptr_t>(X) & 127) != 0) return EJOIN_EINVAL;
  return EJOIN_OK;
}

int ensure_workspace(ejoin_ctx* ctx, int64_t n) {
  if (n <= ctx->s_cap) return EJOIN_OK;
  if (ctx->s) {
    EJ_TRY(hipDeviceSynchronize());
    EJ_TRY(hipFree(ctx->s));
    ctx->s = nullptr;
    ctx->s_cap = 0;
  }
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&ctx->s), (size_t)n * sizeof(float));
  if (e == hipErrorOutOfMemory) {
    (void)hipGetLastError();
    return EJOIN_ENOMEM;
  }
  if (e != hipSuccess) return fail_hip(ctx, e, "hipMalloc(norm workspace)");
  ctx->s_cap = n;
  return EJOIN_OK;
}

int launch_norms(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float* s, hipStream_t st) {
  const int k16 = (d + KSLICE - 1) / KSLICE * (KSLICE / 16);
  const int64_t waves = (n + 31) / 32;
  const unsigned blocks = (unsigned)((waves + 3) / 4);
  hipLaunchKernelGGL(k_norms, dim3(blocks), dim3(256), 0, st, X, n, ld, k16, s);
  EJ_TRY(hipGetLastError());
  return EJOIN_OK;
}

struct DeviceGuard {
  int prev;
  bool ok;
  explicit DeviceGuard(int dev) : prev(-1), ok(false) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
  }
  ~DeviceGuard() {
    int cur = -1;
    if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

template <bool COUNT>
int run_join(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps, uint32_t* pairs, float* dist2,
             uint64_t capacity, uint64_t* n_pairs, uint32_t* counts, uint64_t* total, hipStream_t st) {
  int rc = ensure_workspace(ctx, n);
  if (rc != EJOIN_OK) return rc;
  JoinArgs a;
  memset(&a, 0, sizeof(a));
  a.X = X;
  a.s = ctx->s;
  a.n = n;
  a.ld = ld;
  a.nslices = (d + KSLICE - 1) / KSLICE;
  a.eps2 = eps * eps;
  a.ntiles = (uint32_t)((n + TILE - 1) / TILE);
  a.nsb = (a.ntiles + SB - 1) / SB;
  const uint64_t items = (uint64_t)a.nsb * (a.nsb + 1) / 2 * 32;
  if (items >= 0xFFFFFFFFull - 4096) return EJOIN_EUNSUPPORTED;
  a.items_per_xcd = (uint32_t)items;
  a.queue = ctx->queue;
  a.pairs = pairs;
  a.dist2 = dist2;
  a.capacity = capacity;
  a.n_pairs = reinterpret_cast<unsigned long long*>(n_pairs);
  a.counts = counts;
  a.total = reinterpret_cast<unsigned long long*>(total);

  if (ctx->profiling) EJ_TRY(hipEventRecord(ctx->ev[0], st));
  rc = launch_norms(ctx, X, n, d, ld, ctx->s, st);
  if (rc != EJOIN_OK) return rc;
  if (ctx->profiling) EJ_TRY(hipEventRecord(ctx->ev[1], st));
  hipLaunchKernelGGL(k_reset, dim3(1), dim3(64), 0, st, ctx->queue, COUNT ? a.total : a.n_pairs, (unsigned long long*)nullptr);
  EJ_TRY(hipGetLastError());
  if (COUNT) {
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, counts, n, 0u);
    EJ_TRY(hipGetLastError());
  }
  if (ctx->profiling) EJ_TRY(hipEventRecord(ctx->ev[2], st));
  hipLaunchKernelGGL(k_join<COUNT>, dim3(ctx->num_cu), dim3(THREADS), LDS_BYTES, st, a);
  EJ_TRY(hipGetLastError());
  if (ctx->profiling) {
    EJ_TRY(hipEventRecord(ctx->ev[3], st));
    ctx->ev_valid = 1;
  }
  return EJOIN_OK;
}

}  // namespace

extern "C" {

int ejoin_create(ejoin_ctx** out, int device) {
  if (!out) return EJOIN_EINVAL;
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) {
    (void)hipGetLastError();
    return EJOIN_EINVAL;
  }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) {
    (void)hipGetLastError();
    return EJOIN_EHIP;
  }
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return EJOIN_EUNSUPPORTED;
  ejoin_ctx* ctx = new (std::nothrow) ejoin_ctx();
  if (!ctx) return EJOIN_ENOMEM;
  memset(ctx, 0, sizeof(*ctx));
  ctx->device = device;
  ctx->num_cu = prop.multiProcessorCount;
  DeviceGuard guard(device);
  if (!guard.ok) {
    delete ctx;
    return EJOIN_EHIP;
  }
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&ctx->queue), 256);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->scratch), 256);
  for (int i = 0; i < 4 && e == hipSuccess; ++i) e = hipEventCreate(&ctx->ev[i]);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_join<false>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_join<true>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    ejoin_destroy(ctx);
    return EJOIN_EHIP;
  }
  *out = ctx;
  return EJOIN_OK;
}

int ejoin_destroy(ejoin_ctx* ctx) {
  if (!ctx) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (ctx->queue) (void)hipFree(ctx->queue);
  if (ctx->scratch) (void)hipFree(ctx->scratch);
  if (ctx->s) (void)hipFree(ctx->s);
  for (int i = 0; i < 4; ++i)
    if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
  delete ctx;
  return EJOIN_OK;
}

int ejoin_reserve(ejoin_ctx* ctx, int64_t n) {
  if (!ctx || n < 1) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return ensure_workspace(ctx, n);
}

const char* ejoin_strerror(int code) {
  switch (code) {
    case EJOIN_OK: return "ok";
    case EJOIN_EINVAL: return "invalid argument (null pointer, size out of range, ld not a multiple of 64 or < roundup(d,64), X not 128-byte aligned)";
    case EJOIN_EUNSUPPORTED: return "unsupported device (gfx950 required) or problem size";
    case EJOIN_EHIP: return "HIP runtime error (see ejoin_last_hip_error)";
    case EJOIN_ENOMEM: return "out of device memory for the norm workspace";
    default: return "unknown error code";
  }
}

const char* ejoin_last_hip_error(const ejoin_ctx* ctx) { return ctx ? ctx->hip_error : ""; }

int ejoin_norms(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float* s, void* stream) {
  int rc = check_common(ctx, X, n, d, ld);
  if (rc != EJOIN_OK) return rc;
  if (!s) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return launch_norms(ctx, X, n, d, ld, s, static_cast<hipStream_t>(stream));
}

int ejoin_selfjoin_count(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps, uint32_t* counts,
                         uint64_t* total_pairs, void* stream) {
  int rc = check_common(ctx, X, n, d, ld);
  if (rc != EJOIN_OK) return rc;
  if (!counts || !total_pairs || !(eps >= 0.f) || !isfinite(eps)) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return run_join<true>(ctx, X, n, d, ld, eps, nullptr, nullptr, 0, nullptr, counts, total_pairs, static_cast<hipStream_t>(stream));
}

int ejoin_selfjoin_pairs(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps, uint32_t* pairs,
                         float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream) {
  int rc = check_common(ctx, X, n, d, ld);
  if (rc != EJOIN_OK) return rc;
  if (!n_pairs || (!pairs && capacity > 0) || !(eps >= 0.f) || !isfinite(eps)) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return run_join<false>(ctx, X, n, d, ld, eps, pairs, dist2, capacity, n_pairs, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

int ejoin_dist2_tile(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, int64_t i0, int64_t j0, int32_t rows,
                     int32_t cols, float* out, void* stream) {
  int rc = check_common(ctx, X, n, d, ld);
  if (rc != EJOIN_OK) return rc;
  if (!out || rows < 1 || cols < 1 || i0 < 0 || j0 < 0 || i0 + rows > n || j0 + cols > n) return EJOIN_EINVAL;
  if (rows > 32 * 65535 || cols > 32 * 65535) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  rc = ensure_workspace(ctx, n);
  if (rc != EJOIN_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  rc = launch_norms(ctx, X, n, d, ld, ctx->s, st);
  if (rc != EJOIN_OK) return rc;
  const int k16 = (d + KSLICE - 1) / KSLICE * (KSLICE / 16);
  hipLaunchKernelGGL(k_dist2_tile, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(64), 0, st, X, ctx->s, n, ld, k16, i0, j0, rows, cols, out);
  EJ_TRY(hipGetLastError());
  return EJOIN_OK;
}

int ejoin_set_profiling(ejoin_ctx* ctx, int on) {
  if (!ctx) return EJOIN_EINVAL;
  ctx->profiling = on ? 1 : 0;
  ctx->ev_valid = 0;
  return EJOIN_OK;
}

int ejoin_last_kernel_ms(ejoin_ctx* ctx, float* norms_ms, float* join_ms) {
  if (!ctx || !ctx->ev_valid) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  EJ_TRY(hipEventSynchronize(ctx->ev[3]));
  float a = 0.f, b = 0.f;
  EJ_TRY(hipEventElapsedTime(&a, ctx->ev[0], ctx->ev[1]));
  EJ_TRY(hipEventElapsedTime(&b, ctx->ev[2], ctx->ev[3]));
  if (norms_ms) *norms_ms = a;
  if (join_ms) *join_ms = b;
  return EJOIN_OK;
}

int64_t ejoin_tiles_evaluated(int64_t n) {
  if (n < 1) return 0;
  const int64_t t = (n + TILE - 1) / TILE;
  return t * (t + 1) / 2;
}

}  // extern "C"
