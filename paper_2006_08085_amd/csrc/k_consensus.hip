// The whole factor sequence of the exact average consensus (Lemma 1 of the
// paper; spanning-tree gather and propagate steps) applied on chip, for up to
// 256 workers: Z <- A_{R-1} ... A_0 Z with the state read and written once.
//
// One wavefront owns 64 columns and all n rows of them; the rows sit in LDS
// (n x 64 fp32) and stay there.  A gather or propagate step changes only the
// rows of one level of the tree and their parents; every other row of the factor
// is an identity row and costs nothing, and a changed row that no later step
// reads before it is overwritten again (the emptied rows of the gather steps) is
// dropped on the host.  What remains becomes one list of small operations, four
// to a batch:
//   acc_j = (acc_{j-1} & keep) + w0 * (row[o0] & m0) + w1 * (row[o1] & m1),   row[dst] = acc_j,
// the masks being all ones or zero, so that an absent term is exactly absent
// whatever the row it points at holds.  A row of up to 8 terms is a chain of up
// to 4 operations of one batch, each writing its partial sum to the row, the
// last one last.  The code of a batch has no branch: 32 words fetched with
// scalar loads (the next batch's while this one computes), every operand read
// before any row is written.  Within a step the host orders the rows so that a
// row is overwritten only in or after the batch of its last reader, which is
// what a step of the sequence means (every row is computed from the state
// before the step); a step whose rows cannot be ordered that way (a cycle of
// rows reading each other) is left to the one-launch-per-factor path.
// No wavefront waits for another: there is no barrier.
#include "detag_internal.h"
#include "dev_common.hpp"

namespace detag {
namespace {

constexpr int kCols = 64, kRowsMax = 256, kTerms = 8;
constexpr int kBatch = 4;                      // operations per batch
constexpr int kRowChunk = 64, kRowTail = 16;  // rows loaded or stored together

struct Op {
  uint32_t o0, o1, dst;  // byte offsets of the two source rows and of the written row in the tile (< 65536)
  uint32_t keep;         // all ones: continue the previous operation's sum; 0: start from 0
  uint32_t w0, w1;       // fp32 weights
  uint32_t m0, m1;       // all ones: the term is there; 0: it is not
};
struct BatchWords {
  Op op[kBatch];
};
constexpr int kBatchWords = sizeof(BatchWords) / 4;

__device__ __forceinline__ float masked(float v, uint32_t m) { return __uint_as_float(__float_as_uint(v) & m); }

// One batch on the wavefront's tile; `mine` is the lane's column of row 0.
__device__ __forceinline__ void run_batch(const BatchWords &t, char *mine) {
  float x0[kBatch], x1[kBatch], acc[kBatch];
#pragma unroll
  for (int j = 0; j < kBatch; ++j) {
    x0[j] = *reinterpret_cast<const float *>(mine + t.op[j].o0);
    x1[j] = *reinterpret_cast<const float *>(mine + t.op[j].o1);
  }
#pragma unroll
  for (int j = 0; j < kBatch; ++j) {
    float a = j ? masked(acc[j - 1], t.op[j].keep) : 0.f;
    a = fmaf(__uint_as_float(t.op[j].w0), masked(x0[j], t.op[j].m0), a);
    acc[j] = fmaf(__uint_as_float(t.op[j].w1), masked(x1[j], t.op[j].m1), a);
  }
#pragma unroll
  for (int j = 0; j < kBatch; ++j) *reinterpret_cast<float *>(mine + t.op[j].dst) = acc[j];
}

// The whole table: two batches per trip (the host makes their number even), each fetched while the other one runs.
__device__ __forceinline__ void run_table(const BatchWords *__restrict__ table, int batches, char *mine) {
  BatchWords even = table[0];
  for (int b = 0; b < batches; b += 2) {
    const BatchWords odd = table[b + 1];
    __builtin_amdgcn_sched_barrier(0);
    run_batch(even, mine);
    even = table[b + 2 < batches ? b + 2 : b];
    __builtin_amdgcn_sched_barrier(0);
    run_batch(odd, mine);
  }
}

// CHUNK rows from r0 on, HBM -> LDS, every load issued before the first value is needed.  Rows past the last one
// repeat it (the same value goes to the same place twice), so CHUNK need not divide n.
template <typename ST, int CHUNK>
__device__ __forceinline__ void rows_in_chunk(const ST *Z, int64_t tile, int64_t ld, int n, int r0, uint32_t valid,
                                              uint32_t so, float *col) {
  float v[CHUNK];
#pragma unroll
  for (int k = 0; k < CHUNK; ++k) v[k] = buf_load<ST>(row_of(Z, tile, ld, r0 + k < n ? r0 + k : n - 1, valid), so);
#pragma unroll
  for (int k = 0; k < CHUNK; ++k) col[(r0 + k < n ? r0 + k : n - 1) * kCols] = v[k];
}

template <typename ST, int CHUNK>
__device__ __forceinline__ void rows_out_chunk(ST *Z, int64_t tile, int64_t ld, int n, int r0, uint32_t valid,
                                               uint32_t so, const float *col) {
  float v[CHUNK];
#pragma unroll
  for (int k = 0; k < CHUNK; ++k) v[k] = col[(r0 + k < n ? r0 + k : n - 1) * kCols];
#pragma unroll
  for (int k = 0; k < CHUNK; ++k) buf_store<ST>(row_of(Z, tile, ld, r0 + k < n ? r0 + k : n - 1, valid), so, v[k]);
}

// All n rows of the wavefront's 64 columns: 64 at a time while that many are left, then 16 at a time.
template <typename ST>
__device__ __forceinline__ void rows_in(const ST *Z, int64_t tile, int64_t ld, int n, uint32_t valid, uint32_t so,
                                        float *col) {
  int r0 = 0;
  for (; r0 + kRowChunk <= n; r0 += kRowChunk) rows_in_chunk<ST, kRowChunk>(Z, tile, ld, n, r0, valid, so, col);
  for (; r0 < n; r0 += kRowTail) rows_in_chunk<ST, kRowTail>(Z, tile, ld, n, r0, valid, so, col);
}

template <typename ST>
__device__ __forceinline__ void rows_out(ST *Z, int64_t tile, int64_t ld, int n, uint32_t valid, uint32_t so,
                                         const float *col) {
  int r0 = 0;
  for (; r0 + kRowChunk <= n; r0 += kRowChunk) rows_out_chunk<ST, kRowChunk>(Z, tile, ld, n, r0, valid, so, col);
  for (; r0 < n; r0 += kRowTail) rows_out_chunk<ST, kRowTail>(Z, tile, ld, n, r0, valid, so, col);
}

template <typename ST>
__global__ __launch_bounds__(256) void factor_sequence_kernel(ST *Z, int n, int64_t d, int64_t ld,
                                                              const BatchWords *__restrict__ table, int batches) {
  extern __shared__ float smem[];  // one n x 64 tile per wavefront
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int64_t tile = (int64_t(blockIdx.x) * (blockDim.x >> 6) + w) * kCols;
  if (tile >= d) return;  // no barrier anywhere below
  float *tile_f = smem + size_t(w) * n * kCols;
  char *mine = reinterpret_cast<char *>(tile_f + lane);
  const uint32_t valid = uint32_t(d - tile < kCols ? d - tile : kCols);
  const uint32_t so = lane * uint32_t(sizeof(ST));
  rows_in<ST>(Z, tile, ld, n, valid, so, tile_f + lane);
  run_table(table, batches, mine);
  rows_out<ST>(Z, tile, ld, n, valid, so, tile_f + lane);
}

uint32_t f32_bits(float f) {
  uint32_t u;
  __builtin_memcpy(&u, &f, sizeof u);
  return u;
}

// LDS of a compute unit as far as one block may use it on the current device (queried once).
int max_lds_per_block() {
  static const int bytes = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) {
      (void)hipGetLastError();
      return 0;
    }
    return v;
  }();
  return bytes;
}

struct Row {  // a row of a factor that is not an identity row
  int dst, cnt;
  int col[kTerms];
  float val[kTerms];
};

// Order the changed rows of one step so that whoever reads a row that the step also overwrites comes before (or is)
// the row's writer.  False if they read each other in a cycle.
bool order_rows(int n, std::vector<Row> &rows) {
  const int m = int(rows.size());
  std::vector<int> writer(n, -1), waits(m, 0);
  for (int a = 0; a < m; ++a) writer[rows[a].dst] = a;
  std::vector<std::vector<int>> then(m);  // then[b]: writers that have to come after reader b
  for (int b = 0; b < m; ++b)
    for (int k = 0; k < rows[b].cnt; ++k) {
      const int a = writer[rows[b].col[k]];
      if (a >= 0 && a != b) then[b].push_back(a), ++waits[a];
    }
  std::vector<int> order, ready;
  for (int a = m - 1; a >= 0; --a)
    if (!waits[a]) ready.push_back(a);
  while (!ready.empty()) {
    const int b = ready.back();
    ready.pop_back();
    order.push_back(b);
    for (int a : then[b])
      if (--waits[a] == 0) ready.push_back(a);
  }
  if (int(order.size()) != m) return false;
  std::vector<Row> sorted;
  sorted.reserve(m);
  for (int i : order) sorted.push_back(rows[i]);
  rows.swap(sorted);
  return true;
}

// Drop every changed row whose value nobody uses: going back from the last step, a row is needed after a step if
// it is part of the result or a later kept row reads it before it is written again.
void drop_unused_rows(int n, std::vector<std::vector<Row>> &steps) {
  std::vector<char> needed(n, 1);
  for (size_t s = steps.size(); s-- > 0;) {
    std::vector<Row> kept;
    for (const Row &r : steps[s])
      if (needed[r.dst]) kept.push_back(r);
    for (const Row &r : kept) needed[r.dst] = 0;  // a step reads the state before it, so first the writes...
    for (const Row &r : kept)
      for (int k = 0; k < r.cnt; ++k) needed[r.col[k]] = 1;  // ...then what they read
    steps[s].swap(kept);
  }
}

}  // namespace

// The table is an even number of batches; a batch never holds rows of two steps.
bool build_factor_table(int n, const std::vector<HostFactor> &factors, std::vector<uint32_t> &table) {
  table.clear();
  if (n > kRowsMax) return false;
  std::vector<std::vector<Row>> steps;
  for (const HostFactor &f : factors) {
    std::vector<Row> rows;
    for (int i = 0; i < n; ++i) {
      const int b = f.rowptr[i], cnt = f.rowptr[i + 1] - b;
      if (cnt > kTerms) return false;
      if (cnt == 1 && f.colidx[b] == i && f.vals[b] == 1.0) continue;  // identity row: nothing to do
      Row r{};
      r.dst = i, r.cnt = cnt;
      for (int k = 0; k < cnt; ++k) r.col[k] = f.colidx[b + k], r.val[k] = float(f.vals[b + k]);
      rows.push_back(r);
    }
    steps.push_back(std::move(rows));
  }
  drop_unused_rows(n, steps);
  const auto row_off = [](int i) { return uint32_t(i) * kCols * 4u; };  // byte offset of row i in the tile
  const uint32_t ones = ~0u, one_f = f32_bits(1.f);
  std::vector<Op> ops;
  for (std::vector<Row> &rows : steps) {
    if (!order_rows(n, rows)) return false;
    int room = 0;  // operations left in the open batch
    const auto close_batch = [&] {  // fill up with operations that write the last sum to its row once more
      for (; room > 0 && !ops.empty(); --room) {
        const Op &last = ops.back();
        ops.push_back(Op{last.dst, last.dst, last.dst, ones, 0u, 0u, 0u, 0u});
      }
    };
    for (const Row &r : rows) {
      const int nops = r.cnt > 2 ? (r.cnt + 1) / 2 : 1;
      if (nops > room) close_batch(), room = kBatch;
      for (int o = 0; o < nops; ++o) {
        const int k0 = 2 * o, terms = r.cnt - k0 >= 2 ? 2 : r.cnt - k0;
        Op op{row_off(r.dst), row_off(r.dst), row_off(r.dst), o > 0 ? ones : 0u, 0u, 0u, 0u, 0u};
        if (terms > 0) op.o0 = row_off(r.col[k0]), op.w0 = f32_bits(r.val[k0]), op.m0 = ones;
        if (terms > 1) op.o1 = row_off(r.col[k0 + 1]), op.w1 = f32_bits(r.val[k0 + 1]), op.m1 = ones;
        ops.push_back(op);
      }
      room -= nops;
    }
    close_batch();
  }
  if ((ops.size() / kBatch) % 2) {  // a batch that copies row 0 to itself
    ops.push_back(Op{0u, 0u, 0u, 0u, one_f, 0u, ones, 0u});
    for (int j = 1; j < kBatch; ++j) ops.push_back(Op{0u, 0u, 0u, ones, 0u, 0u, 0u, 0u});
  }
  table.resize(ops.size() * (sizeof(Op) / 4));
  if (!ops.empty()) __builtin_memcpy(table.data(), ops.data(), ops.size() * sizeof(Op));
  return true;
}

// -1: a tile of n rows does not fit the LDS of a block on this device (the caller applies the factors one by one).
int launch_factor_sequence(const Shape &s, const uint32_t *table, int table_words, void *Z, void *stream) {
  const int batches = table_words / kBatchWords;
  if (batches == 0) return 0;  // every row of every factor is an identity row
  const size_t tile_bytes = size_t(s.n) * kCols * sizeof(float), lds_max = size_t(max_lds_per_block());
  // wavefronts per block: whatever keeps most wavefronts on a compute unit, larger blocks on a tie while they
  // stay within the 64 KiB a launch may ask for without raising the kernel's limit
  int waves = 0, resident = 0;
  for (int wv = 1; wv <= 4; wv *= 2) {
    const size_t lds = tile_bytes * wv;
    if (lds > lds_max) break;
    const int res = int(lds_max / lds) * wv;
    if (res > resident || (res == resident && lds <= 65536)) waves = wv, resident = res;
  }
  if (waves == 0) return -1;
  const size_t lds_bytes = tile_bytes * waves;
  const int64_t tiles = ceil_div_i64(s.d, kCols);
  auto st = static_cast<hipStream_t>(stream);
  const auto *tb = reinterpret_cast<const BatchWords *>(table);
  auto launch = [&](auto *kernel, auto *z, int64_t blocks) -> int {
    if (lds_bytes > 65536) {  // above the default limit of a launch: raise it for this kernel
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes));
      if (e != hipSuccess) return hip_rc(e);
    }
    kernel<<<dim3(uint32_t(blocks)), 64 * waves, lds_bytes, st>>>(z, s.n, s.d, s.ld, tb, batches);
    return hip_rc(hipGetLastError());
  };
  const int64_t blocks = (tiles + waves - 1) / waves;
  return s.bf16 ? launch(&factor_sequence_kernel<bf16_t>, static_cast<bf16_t *>(Z), blocks)
                : launch(&factor_sequence_kernel<float>, static_cast<float *>(Z), blocks);
}

}  // namespace detag
