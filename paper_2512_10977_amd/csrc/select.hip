// take, masked_select and nonzero.
//
// take: one lane per output element; the flat index is wrapped and, for a
//   non-contiguous input, decomposed into the input's coordinates.
// masked_select / nonzero: stream compaction in three launches.  The logical
//   index space is cut into tiles of 4096 elements (a 256-lane workgroup; each
//   wave owns 1024 consecutive elements as 16 slabs of 64).
//     count  : every workgroup counts its selected elements (ballot + popcount).
//     offsets: one workgroup turns the counts into exclusive offsets in place
//              and writes the total to the caller's count tensor.
//     write  : every workgroup recomputes its flags; a lane's destination is
//              tile offset + selected elements in earlier waves + earlier
//              slabs + lower lanes of its slab, so the output keeps the
//              logical (row-major) order.
#include <cstring>

#include "common.h"
#include "index_util.h"

namespace tx {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr int kSlabs = 16;                           // slabs of 64 elements per wave
constexpr int kTile = kBlock * kSlabs;               // 4096 elements per workgroup
constexpr int kScanBlock = 1024;




// ---------------------------------------------------------------------------
// take
// ---------------------------------------------------------------------------
struct TakeArgs {
  Dims shape;                        // index's (= out's) shape
  Dims in_shape;                     // input's shape (used when the input is not contiguous)
  int64_t istride[TX_MAX_DIMS], ostride[TX_MAX_DIMS], sstride[TX_MAX_DIMS];
  const char* index;
  const char* src;
  char* dst;
  int64_t in_numel;
  int index_is64, contiguous;
};

constexpr int kTakeU = 4;
template <class B>
__global__ __launch_bounds__(kBlock) void take_kernel(const TakeArgs a) {
  int64_t so[kTakeU], d_o[kTakeU];
  bool live[kTakeU];
#pragma unroll
  for (int u = 0; u < kTakeU; ++u) {
    const int64_t lin = ((int64_t)blockIdx.x * kTakeU + u) * kBlock + threadIdx.x;
    live[u] = lin < a.shape.numel;
    so[u] = d_o[u] = 0;
    if (!live[u]) continue;
    int64_t io = 0;
    uint32_t rem = (uint32_t)lin;
    for (int d = a.shape.n - 1; d >= 0; --d) {
      uint32_t q, m;
      a.shape.div[d].divmod(rem, q, m);
      rem = q;
      io += (int64_t)m * a.istride[d];
      d_o[u] += (int64_t)m * a.ostride[d];
    }
    int64_t k = load_index(a.index, io, a.index_is64);
    k += k < 0 ? a.in_numel : 0;
    if (a.contiguous) {
      so[u] = k;
    } else {
      uint32_t r2 = (uint32_t)k;
      for (int d = a.in_shape.n - 1; d >= 0; --d) {
        uint32_t q, m;
        a.in_shape.div[d].divmod(r2, q, m);
        r2 = q;
        so[u] += (int64_t)m * a.sstride[d];
      }
    }
  }
  B v[kTakeU];
#pragma unroll
  for (int u = 0; u < kTakeU; ++u)
    if (live[u]) v[u] = ((const B*)a.src)[so[u]];
#pragma unroll
  for (int u = 0; u < kTakeU; ++u)
    if (live[u]) ((B*)a.dst)[d_o[u]] = v[u];
}

// ---------------------------------------------------------------------------
// compaction
// ---------------------------------------------------------------------------
struct SelectArgs {
  Dims shape;                        // logical (broadcast) shape that is walked in row-major order
  int64_t fstride[TX_MAX_DIMS];      // strides of the tensor the flags come from (mask, or x for nonzero)
  int64_t pstride[TX_MAX_DIMS];      // masked_select: strides of x
  const char* flag;
  const char* payload;
  char* out;
  int64_t ostride0, ostride1;        // out strides in elements
  int64_t capacity;                  // rows of out
  uint32_t* offsets;                 // per tile: count, then exclusive offset
  int64_t* count;
  int64_t ntiles;
  unsigned long long zmask;          // nonzero: bits of an element that must not all be zero
  int contiguous;                    // flags (and payload) can be addressed by the linear index
};

template <int ES> struct Raw;
template <> struct Raw<1> { using type = uint8_t; };
template <> struct Raw<2> { using type = uint16_t; };
template <> struct Raw<4> { using type = uint32_t; };
template <> struct Raw<8> { using type = unsigned long long; };

// offset of logical element lin in the flag tensor (and in the payload tensor)
__device__ __forceinline__ void select_offsets(const SelectArgs& a, int64_t lin, int64_t* fo, int64_t* po) {
  if (a.contiguous) { *fo = lin; *po = lin; return; }
  int64_t f = 0, p = 0;
  uint32_t rem = (uint32_t)lin;
  for (int d = a.shape.n - 1; d >= 0; --d) {
    uint32_t q, m;
    a.shape.div[d].divmod(rem, q, m);
    rem = q;
    f += (int64_t)m * a.fstride[d];
    p += (int64_t)m * a.pstride[d];
  }
  *fo = f;
  *po = p;
}

// flags of the wave's 16 slabs as ballots.  FES: bytes per flag element.
template <int FES>
__device__ __forceinline__ void slab_ballots(const SelectArgs& a, int64_t wave_base, int lane, unsigned long long (&bal)[kSlabs],
                                             int64_t (&poff)[kSlabs]) {
  using F = typename Raw<FES>::type;
  if constexpr (FES == 1) {
    // one-byte flags addressed linearly: a lane fetches the 16 flags of elements [16 lane, 16 lane + 16) with one
    // 16-byte load (64 one-byte loads per slab would move 64 bytes per instruction) and folds them to 16 bits;
    // slab s is then the concatenation of the masks held by lanes 4s .. 4s + 3
    if (a.contiguous && wave_base + kSlabs * kWave <= a.shape.numel && ((uintptr_t)(a.flag + wave_base) & 15) == 0) {
      const u32x4 v = *(const u32x4*)(a.flag + wave_base + lane * 16);
      uint32_t m16 = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint32_t t = v[q];
        t |= t >> 4;
        t |= t >> 2;
        t |= t >> 1;                                    // bit 8k = byte k is not zero
        m16 |= ((t & 1u) | ((t >> 7) & 2u) | ((t >> 14) & 4u) | ((t >> 21) & 8u)) << (4 * q);
      }
#pragma unroll
      for (int s = 0; s < kSlabs; ++s) {
        unsigned long long b = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          b |= (unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)m16, 4 * s + q) << (16 * q);
        bal[s] = b;
        poff[s] = wave_base + s * kWave + lane;
      }
      return;
    }
  }
  F raw[kSlabs];
#pragma unroll
  for (int s = 0; s < kSlabs; ++s) {
    const int64_t lin = wave_base + s * kWave + lane;
    int64_t fo;
    select_offsets(a, lin < a.shape.numel ? lin : a.shape.numel - 1, &fo, &poff[s]);    // clamped: unconditional load
    raw[s] = ((const F*)a.flag)[fo];
  }
#pragma unroll
  for (int s = 0; s < kSlabs; ++s) {
    const int64_t lin = wave_base + s * kWave + lane;
    const bool on = lin < a.shape.numel && ((unsigned long long)raw[s] & a.zmask) != 0;
    bal[s] = __ballot(on);
  }
}

template <int FES>
__global__ __launch_bounds__(kBlock) void select_count_kernel(const SelectArgs a) {
  __shared__ uint32_t wave_count[kWaves];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t wave_base = (int64_t)blockIdx.x * kTile + (int64_t)w * (kSlabs * kWave);
  unsigned long long bal[kSlabs];
  int64_t poff[kSlabs];
  slab_ballots<FES>(a, wave_base, lane, bal, poff);
  uint32_t c = 0;
#pragma unroll
  for (int s = 0; s < kSlabs; ++s) c += (uint32_t)__popcll(bal[s]);
  if (lane == 0) wave_count[w] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) t += wave_count[i];
    a.offsets[blockIdx.x] = t;
  }
}

// counts -> exclusive offsets in place; total -> *count.  One workgroup; a lane scans 16 consecutive counts per
// step, so 64 Ki tiles (2^28 elements) take four steps.
constexpr int kScanPer = 16;
__global__ __launch_bounds__(kScanBlock) void select_offsets_kernel(uint32_t* counts, int64_t n, int64_t* total) {
  __shared__ uint32_t wave_tot[kScanBlock / kWave];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  uint32_t carry = 0;
  for (int64_t base = 0; base < n; base += (int64_t)kScanBlock * kScanPer) {
    const int64_t i0 = base + (int64_t)threadIdx.x * kScanPer;
    uint32_t v[kScanPer];
    // a lane's 16 counts are four aligned vectors; every load is unconditional (a lane past the end re-reads the
    // first vectors and zeroes them afterwards), so all four are in flight together
    const bool whole = i0 + kScanPer <= n;
    {
      const int64_t ib = whole ? i0 : 0;
      Vec<uint32_t, 4> t[kScanPer / 4];
#pragma unroll
      for (int k = 0; k < kScanPer / 4; ++k) t[k] = vec_load<uint32_t, 4, false>(counts + ib + 4 * k);
#pragma unroll
      for (int k = 0; k < kScanPer; ++k) v[k] = whole ? t[k / 4].v[k % 4] : 0u;
    }
    if (!whole) {
#pragma unroll
      for (int k = 0; k < kScanPer; ++k) v[k] = i0 + k < n ? counts[i0 + k] : 0u;
    }
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < kScanPer; ++k) sum += v[k];
    uint32_t incl = sum;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const uint32_t up = shfl_up(incl, d);
      if (lane >= d) incl += up;
    }
    if (lane == kWave - 1) wave_tot[w] = incl;
    __syncthreads();
    uint32_t before = carry, all = carry;
#pragma unroll
    for (int k = 0; k < kScanBlock / kWave; ++k) {
      if (k == w) before = all;
      all += wave_tot[k];
    }
    uint32_t run = before + incl - sum;
    if (whole) {
      Vec<uint32_t, 4> t[kScanPer / 4];
#pragma unroll
      for (int k = 0; k < kScanPer; ++k) {
        t[k / 4].v[k % 4] = run;
        run += v[k];
      }
#pragma unroll
      for (int k = 0; k < kScanPer / 4; ++k) vec_store<uint32_t, 4, false>(counts + i0 + 4 * k, t[k]);
    } else {
#pragma unroll
      for (int k = 0; k < kScanPer; ++k) {
        if (i0 + k < n) counts[i0 + k] = run;
        run += v[k];
      }
    }
    carry = all;
    __syncthreads();                        // wave_tot is rewritten by the next step
  }
  if (threadIdx.x == 0) *total = (int64_t)carry;
}

// NONZERO = false: copy the payload element (PES bytes); true: write the coordinates as int64
template <int FES, int PES, bool NONZERO>
__global__ __launch_bounds__(kBlock) void select_write_kernel(const SelectArgs a) {
  __shared__ uint32_t wave_count[kWaves];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t wave_base = (int64_t)blockIdx.x * kTile + (int64_t)w * (kSlabs * kWave);
  unsigned long long bal[kSlabs];
  int64_t poff[kSlabs];
  slab_ballots<FES>(a, wave_base, lane, bal, poff);
  uint32_t c = 0;
#pragma unroll
  for (int s = 0; s < kSlabs; ++s) c += (uint32_t)__popcll(bal[s]);
  if (lane == 0) wave_count[w] = c;
  __syncthreads();
  int64_t pos = a.offsets[blockIdx.x];
  for (int i = 0; i < w; ++i) pos += wave_count[i];
  const unsigned long long below = (1ull << lane) - 1ull;
  using P = typename Raw<PES>::type;
  // every payload load is issued before the first store, and unconditionally (poff of a lane past the end is
  // that of the last element): a load under `if (selected)` would be waited for right there, one slab at a time
  P val[kSlabs];
  if constexpr (!NONZERO) {
#pragma unroll
    for (int s = 0; s < kSlabs; ++s) val[s] = ((const P*)a.payload)[poff[s]];
  }
#pragma unroll
  for (int s = 0; s < kSlabs; ++s) {
    if (bal[s] == 0) continue;                                       // wave-uniform
    const bool on = (bal[s] >> lane) & 1ull;
    const int64_t dst = pos + __popcll(bal[s] & below);
    if (on && dst < a.capacity) {
      if constexpr (NONZERO) {
        uint32_t rem = (uint32_t)(wave_base + s * kWave + lane);
        int64_t* row = (int64_t*)a.out + dst * a.ostride0;
        for (int d = a.shape.n - 1; d >= 0; --d) {
          uint32_t q, m;
          a.shape.div[d].divmod(rem, q, m);
          rem = q;
          row[d * a.ostride1] = (int64_t)m;
        }
      } else {
        ((P*)a.out)[dst * a.ostride0] = val[s];
      }
    }
    pos += __popcll(bal[s]);
  }
}

// ---------------------------------------------------------------------------
// contiguous operands: the same tiles, but a lane owns 4 CONSECUTIVE elements ("quad": 256 elements per wave
// instruction, four quads per wave), so flags and payload move as vectors (16 bytes per lane for 4-byte elements)
// instead of one element per lane.  Logical order inside a quad is lane-major, so a lane's destination is the
// quad's base + the selected elements of lower lanes + those of its own lower elements.
// ---------------------------------------------------------------------------
constexpr int kQuads = kSlabs * kWave / (4 * kWave);      // 4

// bit j = element i + j is selected (flag element not zero under zmask)
template <int FES, bool NT>
__device__ __forceinline__ uint32_t quad_flags(const char* flag, int64_t i, unsigned long long zmask) {
  using F = typename Raw<FES>::type;
  const Vec<F, 4> v = vec_load<F, 4, NT>((const F*)flag + i);
  uint32_t f = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) f |= (uint32_t)(((unsigned long long)v.v[j] & zmask) != 0) << j;
  return f;
}

template <int FES>
__global__ __launch_bounds__(kBlock) void select_count_quad_kernel(const SelectArgs a) {
  __shared__ uint32_t wave_count[kWaves];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t wave_base = (int64_t)blockIdx.x * kTile + (int64_t)w * (kSlabs * kWave);
  uint32_t f[kQuads];
#pragma unroll
  for (int q = 0; q < kQuads; ++q) {
    const int64_t i = wave_base + q * (4 * kWave) + lane * 4;                 // numel is a multiple of 4 on this path
    f[q] = quad_flags<FES, false>(a.flag, i < a.shape.numel ? i : 0, a.zmask);   // clamped: unconditional load
    f[q] = i < a.shape.numel ? f[q] : 0u;
  }
  uint32_t c = 0;
#pragma unroll
  for (int q = 0; q < kQuads; ++q) c += (uint32_t)__popc(f[q]);
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) c += shfl_xor(c, m);
  if (lane == 0) wave_count[w] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) t += wave_count[i];
    a.offsets[blockIdx.x] = t;
  }
}

template <int FES, int PES, bool NONZERO>
__global__ __launch_bounds__(kBlock) void select_write_quad_kernel(const SelectArgs a) {
  __shared__ uint32_t wave_count[kWaves];
  using P = typename Raw<PES>::type;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t wave_base = (int64_t)blockIdx.x * kTile + (int64_t)w * (kSlabs * kWave);
  uint32_t f[kQuads];
  Vec<P, 4> pv[kQuads];
#pragma unroll
  for (int q = 0; q < kQuads; ++q) {
    const int64_t i = wave_base + q * (4 * kWave) + lane * 4;
    const int64_t ic = i < a.shape.numel ? i : 0;
    f[q] = quad_flags<FES, true>(a.flag, ic, a.zmask);
    if constexpr (!NONZERO) pv[q] = vec_load<P, 4, true>((const P*)a.payload + ic);
  }
  const unsigned long long below = (1ull << lane) - 1ull;
  uint32_t lane_prefix[kQuads], quad_total[kQuads], c = 0;
#pragma unroll
  for (int q = 0; q < kQuads; ++q) {
    const int64_t i = wave_base + q * (4 * kWave) + lane * 4;
    f[q] = i < a.shape.numel ? f[q] : 0u;
    const uint32_t n = (uint32_t)__popc(f[q]);                              // 0 .. 4: three ballots give the lane prefix
    const unsigned long long b0 = __ballot(n & 1u), b1 = __ballot(n & 2u), b2 = __ballot(n & 4u);
    lane_prefix[q] = (uint32_t)(__popcll(b0 & below) + 2 * __popcll(b1 & below) + 4 * __popcll(b2 & below));
    quad_total[q] = (uint32_t)(__popcll(b0) + 2 * __popcll(b1) + 4 * __popcll(b2));
    c += quad_total[q];
  }
  if (lane == 0) wave_count[w] = c;
  __syncthreads();
  if constexpr (!NONZERO) {
    // The selected elements are first put in output order in LDS, then written by consecutive lanes to consecutive
    // addresses (stored straight from the registers they form four interleaved streams with gaps between the lanes).
    __shared__ P ordered[kTile];
    uint32_t local = 0, total = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
      if (i < w) local += wave_count[i];
      total += wave_count[i];
    }
#pragma unroll
    for (int q = 0; q < kQuads; ++q) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if ((f[q] >> j) & 1u) ordered[local + lane_prefix[q] + __popc(f[q] & ((1u << j) - 1u))] = pv[q].v[j];
      local += quad_total[q];
    }
    __syncthreads();
    const int64_t first = a.offsets[blockIdx.x];
    for (uint32_t i = threadIdx.x; i < total; i += kBlock) {
      const int64_t dst = first + i;
      if (dst < a.capacity) ((P*)a.out)[dst * a.ostride0] = ordered[i];
    }
    return;
  }
  int64_t pos = a.offsets[blockIdx.x];
  for (int i = 0; i < w; ++i) pos += wave_count[i];
#pragma unroll
  for (int q = 0; q < kQuads; ++q) {
    if (quad_total[q] == 0) continue;                                       // wave-uniform
    const int64_t i = wave_base + q * (4 * kWave) + lane * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t dst = pos + lane_prefix[q] + __popc(f[q] & ((1u << j) - 1u));
      if (((f[q] >> j) & 1u) && dst < a.capacity) {
        if constexpr (NONZERO) {
          uint32_t rem = (uint32_t)(i + j);
          int64_t* row = (int64_t*)a.out + dst * a.ostride0;
          for (int d = a.shape.n - 1; d >= 0; --d) {
            uint32_t qq, m;
            a.shape.div[d].divmod(rem, qq, m);
            rem = qq;
            row[d * a.ostride1] = (int64_t)m;
          }
        } else {
          ((P*)a.out)[dst * a.ostride0] = pv[q].v[j];
        }
      }
    }
    pos += quad_total[q];
  }
}

// ---------------------------------------------------------------------------
// single pass: the quad form with the tile's output offset found by decoupled look-back instead of by a count
// pass and an offsets pass (the flags are read once, two launches and the one-workgroup pass fall away).
// Workgroups of 1024 lanes take tiles of 16384 elements in ticket order - with 4096-element tiles the ticket
// counter alone (one same-address atomic per tile, about 12 ns each) would take longer than the copy.  A tile
// publishes its count, then the count of everything up to and including it, as (flag << 32 | count) words; wave 0
// inspects 64 predecessors at a time.  The wait is bounded and sets the header's error word instead of hanging.
// ---------------------------------------------------------------------------
constexpr int kFusedBlock = 1024, kFusedWaves = kFusedBlock / kWave;
constexpr int kFusedQuads = 8;                                     // vectors of 4 elements per lane
constexpr int kFusedTile = kFusedBlock * kFusedQuads * 4;           // 32768
constexpr uint32_t kTileEmpty = 0, kTileAggregate = 1, kTilePrefix = 2;
constexpr int kSelectSpinLimit = 1 << 24;
struct SelectHeader {                                               // first 256 bytes of the workspace
  unsigned int ticket, error;
};

__global__ void select_clear_kernel(unsigned long long* ws, int64_t words) {      // second word: the look-back tag
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < words) ws[i] = i == 1 ? kLookbackMagic : 0ull;
}

template <int FES, int PES>
__global__ __launch_bounds__(kFusedBlock) void select_fused_quad_kernel(const SelectArgs a, int64_t ntiles) {
  __shared__ uint32_t wave_count[kFusedWaves];
  __shared__ unsigned int my_ticket;
  __shared__ uint32_t tile_offset;
  using P = typename Raw<PES>::type;
  SelectHeader* hdr = (SelectHeader*)a.offsets;
  unsigned long long* status = (unsigned long long*)((char*)a.offsets + 256);
  if (threadIdx.x == 0) my_ticket = atomicAdd(&hdr->ticket, 1u);
  __syncthreads();
  const int64_t tile = my_ticket;
  if (tile >= ntiles) return;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t wave_base = tile * kFusedTile + (int64_t)w * (kFusedQuads * 4 * kWave);
  uint32_t f[kFusedQuads];
  Vec<P, 4> pv[kFusedQuads];
#pragma unroll
  for (int q = 0; q < kFusedQuads; ++q) {
    const int64_t i = wave_base + q * (4 * kWave) + lane * 4;
    const int64_t ic = i < a.shape.numel ? i : 0;
    f[q] = quad_flags<FES, true>(a.flag, ic, a.zmask);
    pv[q] = vec_load<P, 4, true>((const P*)a.payload + ic);
  }
  const unsigned long long below = (1ull << lane) - 1ull;
  uint32_t lane_prefix[kFusedQuads], quad_total[kFusedQuads], c = 0;
#pragma unroll
  for (int q = 0; q < kFusedQuads; ++q) {
    const int64_t i = wave_base + q * (4 * kWave) + lane * 4;
    f[q] = i < a.shape.numel ? f[q] : 0u;
    const uint32_t n = (uint32_t)__popc(f[q]);
    const unsigned long long b0 = __ballot(n & 1u), b1 = __ballot(n & 2u), b2 = __ballot(n & 4u);
    lane_prefix[q] = (uint32_t)(__popcll(b0 & below) + 2 * __popcll(b1 & below) + 4 * __popcll(b2 & below));
    quad_total[q] = (uint32_t)(__popcll(b0) + 2 * __popcll(b1) + 4 * __popcll(b2));
    c += quad_total[q];
  }
  if (lane == 0) wave_count[w] = c;
  __syncthreads();
  if (w == 0) {
    uint32_t total = lane < kFusedWaves ? wave_count[lane] : 0u;
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) total += shfl_xor(total, m);
    uint32_t prefix = 0;
    auto publish = [&](uint32_t flag, uint32_t v) {
      __hip_atomic_store(status + tile, ((unsigned long long)flag << 32) | v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    if (tile == 0) {
      if (lane == 0) publish(kTilePrefix, total);
    } else {
      if (lane == 0) publish(kTileAggregate, total);
      int64_t look = tile - 1;
      bool done = false;
      while (!done) {
        const int64_t mine = look - lane;                  // lane i inspects predecessor look - i
        uint32_t val = 0, flag = kTilePrefix;              // before the first tile: an empty prefix
        if (mine >= 0) {
          int spins = 0;
          do {
            const unsigned long long word = __hip_atomic_load(status + mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            flag = (uint32_t)(word >> 32);
            val = (uint32_t)word;
            if (flag != kTileEmpty) break;
            __builtin_amdgcn_s_sleep(2);
          } while (++spins < kSelectSpinLimit);
          if (flag == kTileEmpty) { hdr->error = 1; flag = kTilePrefix; val = 0; }
        }
        const unsigned long long has_prefix = __ballot(flag == kTilePrefix);
        const int stop = __ffsll((long long)has_prefix) - 1;             // nearest predecessor holding a full prefix
        uint32_t contrib = (mine >= 0 && (stop < 0 || lane <= stop)) ? val : 0u;
#pragma unroll
        for (int m = kWave / 2; m >= 1; m >>= 1) contrib += shfl_xor(contrib, m);
        prefix += contrib;
        if (stop >= 0) done = true;
        else look -= kWave;
      }
      if (lane == 0) publish(kTilePrefix, prefix + total);
    }
    if (lane == 0) {
      tile_offset = prefix;
      if (tile == ntiles - 1) *a.count = (int64_t)prefix + (int64_t)total;
    }
  }
  __syncthreads();
  int64_t pos = tile_offset;
  for (int i = 0; i < w; ++i) pos += wave_count[i];
#pragma unroll
  for (int q = 0; q < kFusedQuads; ++q) {
    if (quad_total[q] == 0) continue;                                       // wave-uniform
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t dst = pos + lane_prefix[q] + __popc(f[q] & ((1u << j) - 1u));
      if (((f[q] >> j) & 1u) && dst < a.capacity) ((P*)a.out)[dst * a.ostride0] = pv[q].v[j];
    }
    pos += quad_total[q];
  }
}

// nonzero in one pass: the flags are read once (for nonzero they are the input itself, so the count pass of the
// three-pass form costs a whole read of x), the tile's output offset comes from the same look-back as above, and the
// coordinates are written by consecutive lanes to consecutive output rows: every wave first parks the tile-local
// index of each of its non-zero elements in LDS, in output order (16 bits each: a wave covers 2048 elements), and
// then walks that list 64 entries at a time.  With two coordinates per row and dense rows a lane's row is one
// 16-byte store.  (The quad form of the three-pass write kernel, whose lanes each store the rows of their own
// four elements, wrote four interleaved streams: 1013 us against 758 us for one element per lane.)
typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
template <int FES>
__global__ __launch_bounds__(kFusedBlock) void nonzero_fused_kernel(const SelectArgs a, int64_t ntiles, int pair_rows) {
  constexpr int kPerWave = kFusedQuads * 4 * kWave;                      // 2048
  __shared__ uint32_t wave_count[kFusedWaves];
  __shared__ unsigned int my_ticket;
  __shared__ uint32_t tile_offset;
  __shared__ uint16_t ids[kFusedWaves][kPerWave];
  SelectHeader* hdr = (SelectHeader*)a.offsets;
  unsigned long long* status = (unsigned long long*)((char*)a.offsets + 256);
  if (threadIdx.x == 0) my_ticket = atomicAdd(&hdr->ticket, 1u);
  __syncthreads();
  const int64_t tile = my_ticket;
  if (tile >= ntiles) return;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t wave_base = tile * kFusedTile + (int64_t)w * kPerWave;
  uint32_t f[kFusedQuads];
#pragma unroll
  for (int q = 0; q < kFusedQuads; ++q) {
    const int64_t i = wave_base + q * (4 * kWave) + lane * 4;
    f[q] = quad_flags<FES, true>(a.flag, i < a.shape.numel ? i : 0, a.zmask);      // clamped: unconditional load
  }
  const unsigned long long below = (1ull << lane) - 1ull;
  uint32_t c = 0;
#pragma unroll
  for (int q = 0; q < kFusedQuads; ++q) {
    const int64_t i = wave_base + q * (4 * kWave) + lane * 4;
    f[q] = i < a.shape.numel ? f[q] : 0u;
    const uint32_t n = (uint32_t)__popc(f[q]);
    const unsigned long long b0 = __ballot(n & 1u), b1 = __ballot(n & 2u), b2 = __ballot(n & 4u);
    const uint32_t lane_prefix = (uint32_t)(__popcll(b0 & below) + 2 * __popcll(b1 & below) + 4 * __popcll(b2 & below));
    const uint32_t quad_total = (uint32_t)(__popcll(b0) + 2 * __popcll(b1) + 4 * __popcll(b2));
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if ((f[q] >> j) & 1u) ids[w][c + lane_prefix + __popc(f[q] & ((1u << j) - 1u))] = (uint16_t)(q * (4 * kWave) + lane * 4 + j);
    c += quad_total;
  }
  if (lane == 0) wave_count[w] = c;
  __syncthreads();
  if (w == 0) {
    uint32_t total = lane < kFusedWaves ? wave_count[lane] : 0u;
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) total += shfl_xor(total, m);
    uint32_t prefix = 0;
    auto publish = [&](uint32_t flag, uint32_t v) {
      __hip_atomic_store(status + tile, ((unsigned long long)flag << 32) | v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    if (tile == 0) {
      if (lane == 0) publish(kTilePrefix, total);
    } else {
      if (lane == 0) publish(kTileAggregate, total);
      int64_t look = tile - 1;
      bool done = false;
      while (!done) {
        const int64_t mine = look - lane;                  // lane i inspects predecessor look - i
        uint32_t val = 0, flag = kTilePrefix;              // before the first tile: an empty prefix
        if (mine >= 0) {
          int spins = 0;
          do {
            const unsigned long long word = __hip_atomic_load(status + mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            flag = (uint32_t)(word >> 32);
            val = (uint32_t)word;
            if (flag != kTileEmpty) break;
            __builtin_amdgcn_s_sleep(2);
          } while (++spins < kSelectSpinLimit);
          if (flag == kTileEmpty) { hdr->error = 1; flag = kTilePrefix; val = 0; }
        }
        const unsigned long long has_prefix = __ballot(flag == kTilePrefix);
        const int stop = __ffsll((long long)has_prefix) - 1;             // nearest predecessor holding a full prefix
        uint32_t contrib = (mine >= 0 && (stop < 0 || lane <= stop)) ? val : 0u;
#pragma unroll
        for (int m = kWave / 2; m >= 1; m >>= 1) contrib += shfl_xor(contrib, m);
        prefix += contrib;
        if (stop >= 0) done = true;
        else look -= kWave;
      }
      if (lane == 0) publish(kTilePrefix, prefix + total);
    }
    if (lane == 0) {
      tile_offset = prefix;
      if (tile == ntiles - 1) *a.count = (int64_t)prefix + (int64_t)total;
    }
  }
  __syncthreads();
  int64_t pos = tile_offset;
  for (int i = 0; i < w; ++i) pos += wave_count[i];
  for (uint32_t t = lane; t < c; t += kWave) {
    const int64_t dst = pos + t;
    if (dst >= a.capacity) break;                          // later entries of this lane lie further on still
    uint32_t rem = (uint32_t)(wave_base + ids[w][t]);
    if (pair_rows) {
      uint32_t q, m;
      a.shape.div[1].divmod(rem, q, m);
      const u64x2 row = {(unsigned long long)q, (unsigned long long)m};
      __builtin_nontemporal_store(row, (u64x2*)a.out + dst);
    } else {
      int64_t* row = (int64_t*)a.out + dst * a.ostride0;
      for (int d = a.shape.n - 1; d >= 0; --d) {
        uint32_t q, m;
        a.shape.div[d].divmod(rem, q, m);
        rem = q;
        row[d * a.ostride1] = (int64_t)m;
      }
    }
  }
}

inline int64_t fused_tiles(int64_t n) { return (n + kFusedTile - 1) / kFusedTile; }
inline size_t fused_ws_bytes(int64_t n) { return 256 + (size_t)fused_tiles(n) * 8; }

template <int FES, int PES, bool NONZERO>
tx_status run_select(SelectArgs& a, void* ws, hipStream_t stream) {
  a.offsets = (uint32_t*)ws;
  // vector ("quad") kernels: linear addressing, whole vectors of 4 elements, aligned bases
  const size_t fal = std::min<size_t>(16, 4 * FES), pal = std::min<size_t>(16, 4 * PES);
  const bool quad = a.contiguous && a.shape.numel % 4 == 0 && (uintptr_t)a.flag % fal == 0 &&
                    (NONZERO || (uintptr_t)a.payload % pal == 0) && strcmp(forced_path(), "select-slab") != 0;
  const dim3 grid((unsigned)a.ntiles);
  if constexpr (!NONZERO) {
    // an alternative kept for comparison: on [1048576,256] fp32 at 30 % selected it measured 391 us against 370 us
    // for the three passes (count 67, offsets 20, write 281) - what the look-back costs a 1024-lane workgroup that
    // holds its tile in registers meanwhile is more than the second read of the mask (the fp32 instance needs 78
    // vector registers, so a CU holds one such workgroup; capped at 64 it spills 20 of them and takes 708 us)
    if (quad && a.shape.numel > 0 && !strcmp(forced_path(), "select-fused")) {
      const int64_t ntiles = fused_tiles(a.shape.numel);
      const int64_t words = (int64_t)(fused_ws_bytes(a.shape.numel) / 8);
      hipLaunchKernelGGL(select_clear_kernel, dim3((unsigned)((words + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream,
                         (unsigned long long*)ws, words);
      hipLaunchKernelGGL((select_fused_quad_kernel<FES, PES>), dim3((unsigned)ntiles), dim3(kFusedBlock), 0, stream, a, ntiles);
      set_path("select-fused");
      return check_launch("single-pass compaction kernel");
    }
  }
  if constexpr (NONZERO) {
    // the input is its own flag tensor here, so the single pass saves a whole read of it ("select-3pass" keeps the
    // count, offsets and write kernels)
    if (quad && a.shape.numel > 0 && strcmp(forced_path(), "select-3pass") != 0) {
      const int64_t ntiles = fused_tiles(a.shape.numel);
      const int64_t words = (int64_t)(fused_ws_bytes(a.shape.numel) / 8);
      const int pair_rows = a.shape.n == 2 && a.ostride0 == 2 && a.ostride1 == 1 && (uintptr_t)a.out % 16 == 0;
      hipLaunchKernelGGL(select_clear_kernel, dim3((unsigned)((words + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream,
                         (unsigned long long*)ws, words);
      hipLaunchKernelGGL((nonzero_fused_kernel<FES>), dim3((unsigned)ntiles), dim3(kFusedBlock), 0, stream, a, ntiles, pair_rows);
      set_path("nonzero-fused");
      return check_launch("single-pass nonzero kernel");
    }
  }
  if (a.shape.numel > 0) {
    if (quad) hipLaunchKernelGGL((select_count_quad_kernel<FES>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((select_count_kernel<FES>), grid, dim3(kBlock), 0, stream, a);
  }
  hipLaunchKernelGGL(select_offsets_kernel, dim3(1), dim3(kScanBlock), 0, stream, a.offsets, a.ntiles, a.count);
  if (a.shape.numel > 0) {
    // coordinates (nonzero) are written by the element-per-lane form either way: there consecutive lanes write
    // consecutive output rows, while the quad form scatters four interleaved store streams (measured 1013 us
    // against 758 us on [1048576,256] fp32 at 30 % non-zero)
    if (quad && !NONZERO) hipLaunchKernelGGL((select_write_quad_kernel<FES, PES, false>), grid, dim3(kBlock), 0, stream, a);
    else hipLaunchKernelGGL((select_write_kernel<FES, PES, NONZERO>), grid, dim3(kBlock), 0, stream, a);
  }
  if (a.contiguous && !quad) set_path("select-slab");
  return check_launch("compaction kernels");
}

bool row_major(const tx_tensor* t) {
  int64_t expect = 1;
  for (int d = t->ndim - 1; d >= 0; --d) {
    if (t->sizes[d] != 1 && t->strides[d] != expect) return false;
    expect *= t->sizes[d];
  }
  return true;
}

tx_status count_checks(const tx_tensor* count) {
  tx_status rc;
  if ((rc = check_tensor(count, "count"))) return rc;
  if (count->dtype != TX_I64) return fail(TX_ERR_DTYPE, "count must be int64");
  if (numel(count) != 1) return fail(TX_ERR_SHAPE, "count must hold one element");
  return TX_OK;
}

tx_status ws_checks(const char* name, void* ws, size_t ws_bytes, size_t need) {
  if (!ws || ws_bytes < need) return fail(TX_ERR_WORKSPACE, "%s needs %zu workspace bytes, got %zu", name, need, ws_bytes);
  if ((uintptr_t)ws % 16) return fail(TX_ERR_WORKSPACE, "%s workspace must be 16-byte aligned", name);
  return TX_OK;
}

// the larger of the two forms' needs (per-tile counts of the three-pass form, status words of the single-pass form)
size_t select_ws_bytes(int64_t n) { return std::max((size_t)((n + kTile - 1) / kTile + 1) * sizeof(uint32_t), fused_ws_bytes(n)); }

tx_status masked_select_checks(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x, const tx_tensor* mask, int* nd,
                               int64_t* shape) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x")) || (rc = check_tensor(mask, "mask")) ||
      (rc = count_checks(count)))
    return rc;
  if (mask->dtype != TX_BOOL) return fail(TX_ERR_DTYPE, "masked_select: mask must be bool");
  if (out->dtype != x->dtype) return fail(TX_ERR_DTYPE, "masked_select: out must have x's dtype");
  if (out->ndim != 1) return fail(TX_ERR_SHAPE, "masked_select: out is a 1-D buffer");
  const tx_tensor* ins[2] = {x, mask};
  if ((rc = broadcast_shapes(ins, 2, nd, shape))) return rc;
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  for (const tx_tensor* in : {x, mask, count})
    if (numel(out) && numel(in) && (partial_overlap(out, in) || out->data == in->data))
      return fail(TX_ERR_OVERLAP, "masked_select: out overlaps an input");
  return TX_OK;
}

tx_status nonzero_checks(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(x, "x")) || (rc = count_checks(count))) return rc;
  if (out->dtype != TX_I64) return fail(TX_ERR_DTYPE, "nonzero: out must be int64");
  if (out->ndim != 2 || out->sizes[1] != x->ndim) return fail(TX_ERR_SHAPE, "nonzero: out must be [capacity, x.ndim]");
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  for (const tx_tensor* in : {x, count})
    if (numel(out) && numel(in) && (partial_overlap(out, in) || out->data == in->data))
      return fail(TX_ERR_OVERLAP, "nonzero: out overlaps an input");
  return TX_OK;
}

}  // namespace
}  // namespace tx

using namespace tx;

extern "C" {

tx_status tx_take(const tx_tensor* out, const tx_tensor* input, const tx_tensor* index, void* stream) {
  tx_status rc;
  if ((rc = check_tensor(out, "out")) || (rc = check_tensor(input, "input")) || (rc = check_tensor(index, "index"))) return rc;
  if (index->dtype != TX_I32 && index->dtype != TX_I64) return fail(TX_ERR_DTYPE, "index must be int32 or int64");
  if (out->dtype != input->dtype) return fail(TX_ERR_DTYPE, "take: out must have input's dtype");
  if (!same_sizes(out, index->ndim, index->sizes)) return fail(TX_ERR_SHAPE, "take: out must have index's shape");
  if (!no_internal_overlap(out)) return fail(TX_ERR_OVERLAP, "out has overlapping elements");
  if (numel(out) && ((numel(input) && (partial_overlap(out, input) || out->data == input->data)) || partial_overlap(out, index) ||
                     out->data == index->data))
    return fail(TX_ERR_OVERLAP, "take: out overlaps an input");
  set_path("");
  const int64_t n = numel(out);
  if (n == 0) return TX_OK;
  if (numel(input) == 0) return fail(TX_ERR_INDEX, "take: index into an empty tensor");
  if (n >= (1ll << 31) || numel(input) >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "take: more than 2^31 elements");
  if (index_validation_on() && (rc = validate_index(index, -numel(input), numel(input), "take", as_stream(stream)))) return rc;
  TakeArgs a;
  memset(&a, 0, sizeof(a));
  fill_dims(&a.shape, index->ndim, index->sizes);
  fill_dims(&a.in_shape, input->ndim, input->sizes);
  for (int d = 0; d < index->ndim; ++d) {
    a.istride[d] = index->strides[d];
    a.ostride[d] = out->strides[d];
  }
  for (int d = 0; d < input->ndim; ++d) a.sstride[d] = input->strides[d];
  a.index = (const char*)index->data;
  a.src = (const char*)input->data;
  a.dst = (char*)out->data;
  a.in_numel = numel(input);
  a.index_is64 = index->dtype == TX_I64;
  a.contiguous = row_major(input);
  const dim3 grid((unsigned)((n + kBlock * kTakeU - 1) / (kBlock * kTakeU)));
  hipStream_t s = as_stream(stream);
  set_path(a.contiguous ? "take" : "take-strided");
  switch (dtype_size(input->dtype)) {
    case 1: hipLaunchKernelGGL((take_kernel<uint8_t>), grid, dim3(kBlock), 0, s, a); break;
    case 2: hipLaunchKernelGGL((take_kernel<uint16_t>), grid, dim3(kBlock), 0, s, a); break;
    case 4: hipLaunchKernelGGL((take_kernel<uint32_t>), grid, dim3(kBlock), 0, s, a); break;
    default: hipLaunchKernelGGL((take_kernel<uint64_t>), grid, dim3(kBlock), 0, s, a); break;
  }
  return check_launch("take kernel");
}

size_t tx_masked_select_workspace_bytes(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x, const tx_tensor* mask) {
  int nd;
  int64_t shape[TX_MAX_DIMS];
  if (masked_select_checks(out, count, x, mask, &nd, shape)) return 0;
  int64_t n = 1;
  for (int d = 0; d < nd; ++d) n *= shape[d];
  return select_ws_bytes(n);
}

tx_status tx_masked_select(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x, const tx_tensor* mask,
                           void* workspace, size_t workspace_bytes, void* stream) {
  int nd;
  int64_t shape[TX_MAX_DIMS];
  tx_status rc = masked_select_checks(out, count, x, mask, &nd, shape);
  if (rc) return rc;
  set_path("");
  SelectArgs a;
  memset(&a, 0, sizeof(a));
  fill_dims(&a.shape, nd, shape);
  if (a.shape.numel >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "masked_select: more than 2^31 elements");
  if ((rc = ws_checks("masked_select", workspace, workspace_bytes, select_ws_bytes(a.shape.numel)))) return rc;
  for (int d = 0; d < nd; ++d) {
    const int dm = d - (nd - mask->ndim), dx = d - (nd - x->ndim);
    a.fstride[d] = dm >= 0 && mask->sizes[dm] != 1 ? mask->strides[dm] : 0;
    a.pstride[d] = dx >= 0 && x->sizes[dx] != 1 ? x->strides[dx] : 0;
  }
  a.flag = (const char*)mask->data;
  a.payload = (const char*)x->data;
  a.out = (char*)out->data;
  a.ostride0 = out->strides[0];
  a.capacity = out->sizes[0];
  a.count = (int64_t*)count->data;
  a.ntiles = (a.shape.numel + kTile - 1) / kTile;
  a.zmask = 0xffull;
  a.contiguous = same_sizes(x, nd, shape) && same_sizes(mask, nd, shape) && row_major(x) && row_major(mask);
  hipStream_t s = as_stream(stream);
  set_path(a.contiguous ? "select" : "select-strided");
  switch (dtype_size(x->dtype)) {
    case 1: return run_select<1, 1, false>(a, workspace, s);
    case 2: return run_select<1, 2, false>(a, workspace, s);
    case 4: return run_select<1, 4, false>(a, workspace, s);
    default: return run_select<1, 8, false>(a, workspace, s);
  }
}

size_t tx_nonzero_workspace_bytes(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x) {
  if (nonzero_checks(out, count, x)) return 0;
  return select_ws_bytes(numel(x));
}

tx_status tx_nonzero(const tx_tensor* out, const tx_tensor* count, const tx_tensor* x, void* workspace, size_t workspace_bytes,
                     void* stream) {
  tx_status rc = nonzero_checks(out, count, x);
  if (rc) return rc;
  set_path("");
  SelectArgs a;
  memset(&a, 0, sizeof(a));
  fill_dims(&a.shape, x->ndim, x->sizes);
  if (a.shape.numel >= (1ll << 31)) return fail(TX_ERR_UNSUPPORTED, "nonzero: more than 2^31 elements");
  if ((rc = ws_checks("nonzero", workspace, workspace_bytes, select_ws_bytes(a.shape.numel)))) return rc;
  for (int d = 0; d < x->ndim; ++d) a.fstride[d] = x->strides[d];
  a.flag = (const char*)x->data;
  a.out = (char*)out->data;
  a.ostride0 = out->strides[0];
  a.ostride1 = out->strides[1];
  a.capacity = out->sizes[0];
  a.count = (int64_t*)count->data;
  a.ntiles = (a.shape.numel + kTile - 1) / kTile;
  // floats: every bit but the sign (so -0.0 is zero and a NaN is not); integers and bool: every bit
  a.zmask = x->dtype == TX_F32 ? 0x7fffffffull : dtype_is_float(x->dtype) ? 0x7fffull : ~0ull;
  a.contiguous = row_major(x);
  hipStream_t s = as_stream(stream);
  set_path(a.contiguous ? "select" : "select-strided");
  switch (dtype_size(x->dtype)) {
    case 1: return run_select<1, 8, true>(a, workspace, s);
    case 2: return run_select<2, 8, true>(a, workspace, s);
    case 4: return run_select<4, 8, true>(a, workspace, s);
    default: return run_select<8, 8, true>(a, workspace, s);
  }
}

}  // extern "C"
