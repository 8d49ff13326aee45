// SpMM in "sweep" form, for dense-ish graphs whose gathered operand X is much larger than L2.
//
// Why: the gather  Y[i,:] += val * X[col,:]  is served at L2 speed only while the rows of X it
// touches stay cached.  Cutting the column range into P panels and finishing one panel before the
// next keeps everything in flight inside 1/P of X (the "blocking effect" the paper reports for
// column tiles; the same algebra as its stage loop C += A^{ij} H^j).  Run as P separate launches
// that costs a read-modify-write of Y per panel and a task per (row, panel).  Here instead:
//   - rows are dealt to teams of R rows with equal entry totals (longest first, serpentine), and
//     rows longer than a cap are cut into pieces that become rows of their own, so every team
//     has the same amount of work and therefore advances through the panels at the same pace;
//   - each team's entries are stored contiguously, ordered by (panel, row of the team, column),
//     with the local row in the top bits of the column word: a team is one coalesced stream,
//     no per-row bookkeeping, and the stream prefetch never stalls on a row boundary;
//   - the team keeps its R output rows in LDS for the whole sweep (one private slot per lane,
//     no synchronisation) and writes each row of Y exactly once, with beta and the epilogue.
// The order of additions is fixed by the stored stream, so results are reproducible bit for bit.
#include "common.h"
#include "graph.h"
#include "spmm_device.h"

#include <algorithm>
#include <numeric>
#include <vector>

namespace mggcn {

void build_sweep_set(SweepSet* ss, int32_t n_rows, int32_t n_cols, const int32_t* rowptr, const int32_t* colidx,
                     const float* val, int32_t n_panels, int32_t rows_per_team) {
  const int32_t P = std::max(n_panels, 1);
  const int32_t R = std::min(std::max(rows_per_team, 1), 1 << kSweepRowBits);
  const int64_t nnz = rowptr[n_rows];
  const int64_t width = ceil_div(std::max(n_cols, 1), P);
  ss->n_panels = P;
  ss->R = R;

  // pieces: (row, piece index, pieces of that row, length); long rows are cut so that no piece
  // exceeds about half a team's share
  struct Piece { int32_t row, v, V, len; };
  const int64_t avg = n_rows > 0 ? nnz / n_rows : 0;
  const int64_t cap = std::max<int64_t>(256, (int64_t)R * avg / 2);
  std::vector<Piece> pieces;
  pieces.reserve((size_t)n_rows + (size_t)(nnz / cap) + 16);
  ss->fix.clear();
  int64_t n_partial = 0;
  std::vector<int32_t> first_partial((size_t)n_rows, -1);
  for (int32_t i = 0; i < n_rows; ++i) {
    const int32_t len = rowptr[(size_t)i + 1] - rowptr[i];
    const int32_t V = (int32_t)std::max<int64_t>(1, ceil_div(len, cap));
    if (V > 1) {
      first_partial[i] = (int32_t)n_partial;
      ss->fix.push_back({i, (int32_t)n_partial, V, kTaskFirst | kTaskLast});
      n_partial += V;
    }
    for (int32_t v = 0; v < V; ++v) {
      const int32_t lo = (int32_t)((int64_t)len * v / V), hi = (int32_t)((int64_t)len * (v + 1) / V);
      pieces.push_back({i, v, V, hi - lo});
    }
  }
  ss->n_slots = n_partial;

  // longest first, dealt to the teams in serpentine order: equal totals per team
  std::vector<int64_t> order(pieces.size());
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return pieces[a].len > pieces[b].len; });
  int64_t n_teams = std::max<int64_t>(1, ceil_div((int64_t)pieces.size(), R));
  const int64_t n_teams_padded = ceil_div(n_teams, kSweepTeamPad) * kSweepTeamPad;
  ss->n_teams = n_teams_padded;
  ss->slot_row.assign((size_t)(n_teams_padded * R), -1);
  ss->slot_out.assign((size_t)(n_teams_padded * R), -1);
  std::vector<int64_t> slot_piece((size_t)(n_teams_padded * R), -1);
  for (int64_t k = 0; k < (int64_t)order.size(); ++k) {
    const int64_t round = k / n_teams, pos = k % n_teams;
    const int64_t team = (round & 1) ? (n_teams - 1 - pos) : pos;
    const size_t slot = (size_t)(team * R + round);
    const Piece& pc = pieces[(size_t)order[(size_t)k]];
    slot_piece[slot] = order[(size_t)k];
    ss->slot_row[slot] = pc.row;
    ss->slot_out[slot] = pc.V > 1 ? first_partial[pc.row] + pc.v : -1;
  }

  // per-team streams: panel-major, then local row, then column
  ss->scol.resize((size_t)nnz);
  ss->sval.resize((size_t)nnz);
  ss->team_begin.assign((size_t)n_teams_padded + 1, 0);
  std::vector<int32_t> cut((size_t)R * ((size_t)P + 1));
  int64_t w = 0;
  for (int64_t t = 0; t < n_teams_padded; ++t) {
    ss->team_begin[(size_t)t] = (int32_t)w;
    for (int32_t r = 0; r < R; ++r) {
      int32_t* c = cut.data() + (size_t)r * ((size_t)P + 1);
      const int64_t pi = slot_piece[(size_t)(t * R + r)];
      if (pi < 0) {
        std::fill(c, c + P + 1, 0);
        continue;
      }
      const Piece& pc = pieces[(size_t)pi];
      const int32_t b = rowptr[pc.row], e = rowptr[(size_t)pc.row + 1];
      // panel cuts of the whole row, then this piece's slice of every panel's range
      int32_t prev = b;
      for (int32_t p = 0; p <= P; ++p) {
        const int32_t full = (p == P) ? e
                                      : (int32_t)(std::lower_bound(colidx + prev, colidx + e,
                                                                   (int32_t)std::min<int64_t>(p * width, n_cols)) - colidx);
        c[p] = full;
        prev = full;
      }
    }
    for (int32_t p = 0; p < P; ++p)
      for (int32_t r = 0; r < R; ++r) {
        const int64_t pi = slot_piece[(size_t)(t * R + r)];
        if (pi < 0) continue;
        const Piece& pc = pieces[(size_t)pi];
        const int32_t* c = cut.data() + (size_t)r * ((size_t)P + 1);
        const int32_t lo = c[p], len = c[p + 1] - lo;
        const int32_t s0 = lo + (int32_t)((int64_t)len * pc.v / pc.V), s1 = lo + (int32_t)((int64_t)len * (pc.v + 1) / pc.V);
        for (int32_t k = s0; k < s1; ++k) {
          ss->scol[(size_t)w] = (uint32_t)colidx[k] | ((uint32_t)r << (32 - kSweepRowBits));
          ss->sval[(size_t)w] = val[k];
          ++w;
        }
      }
  }
  ss->team_begin[(size_t)n_teams_padded] = (int32_t)w;
}

namespace {

constexpr int kThreads = 256;

// One team = LPR lanes x VW floats covering a feature chunk; 64/LPR teams per wavefront.
template <int VW, int LPR, int R>
__global__ __launch_bounds__(kThreads) void spmm_sweep(
    const int32_t* __restrict__ team_begin, const uint32_t* __restrict__ scol, const float* __restrict__ sval,
    const int32_t* __restrict__ slot_row, const int32_t* __restrict__ slot_out, const float* __restrict__ X,
    uint32_t ldx_bytes, int F, int n_chunks, float beta, int epi, float* __restrict__ Y, int64_t ldy,
    float* __restrict__ partial, int64_t ldp) {
  constexpr int TPW = 64 / LPR;
  constexpr int U = LPR < 8 ? LPR : 8;
  __shared__ __attribute__((aligned(16))) float rows[(kThreads / 64) * R * 64 * VW];

  const int chunk = (int)(blockIdx.x % (unsigned)n_chunks);
  const int64_t tb = blockIdx.x / (unsigned)n_chunks;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int team = lane / LPR, fl = lane % LPR;
  const int team_base = team * LPR;
  const int64_t T = (tb * (kThreads / 64) + wave) * TPW + team;  // < n_teams: the table is padded

  const int32_t s = team_begin[T];
  const int len = team_begin[T + 1] - s;
  int maxlen = len, minlen = len;
#pragma unroll
  for (int d = LPR; d < 64; d <<= 1) {
    maxlen = max(maxlen, __shfl_xor(maxlen, d));
    minlen = min(minlen, __shfl_xor(minlen, d));
  }
  maxlen = __builtin_amdgcn_readfirstlane(maxlen);
  minlen = __builtin_amdgcn_readfirstlane(minlen);

  const int f0 = chunk * (LPR * VW) + fl * VW;
  const int nf = min(VW, max(0, F - f0));
  const bool live = nf > 0;
  const char* __restrict__ xbase = reinterpret_cast<const char*>(X + f0);
  const uint32_t* __restrict__ cptr = scol + s + fl;
  const float* __restrict__ vptr = sval + s + fl;

  // this lane's private slot of local row r
  float* mine = rows + ((size_t)wave * R * 64 + lane) * VW;
  constexpr int kRowStride = 64 * VW;
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int i = 0; i < VW; ++i) mine[r * kRowStride + i] = 0.f;

  float acc[VW];
  float xs[U][VW];
#pragma unroll
  for (int i = 0; i < VW; ++i) acc[i] = 0.f;
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int i = 0; i < VW; ++i) xs[u][i] = 0.f;
  int cur = 0;  // local row the register accumulator belongs to

  auto flush = [&](int r) {
    float* dst = mine + r * kRowStride;
#pragma unroll
    for (int i = 0; i < VW; ++i) {
      dst[i] += acc[i];
      acc[i] = 0.f;
    }
  };

  uint32_t cw = 0;
  float v = 0.f;
  if (fl < len) {
    cw = __builtin_nontemporal_load(cptr);
    v = __builtin_nontemporal_load(vptr);
  }
  for (int base = 0; base < maxlen; base += LPR) {
    uint32_t cw_next = 0;
    float v_next = 0.f;
    if (base + LPR + fl < len) {
      cw_next = __builtin_nontemporal_load(cptr + base + LPR);
      v_next = __builtin_nontemporal_load(vptr + base + LPR);
    }
    const bool full = base + LPR <= minlen;  // every team of the wavefront has LPR more entries
    const int remaining = maxlen - base;
#pragma unroll 1
    for (int j0 = 0; j0 < LPR; j0 += U) {
      if (j0 >= remaining) break;
      uint32_t cj[U];
      float vs[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        cj[u] = (uint32_t)__shfl((int)cw, team_base + j0 + u);
        vs[u] = __shfl(v, team_base + j0 + u);  // 0 beyond the team's end
      }
      if (full) {
        if (live) {
#pragma unroll
          for (int u = 0; u < U; ++u)
            load_vec<VW>(reinterpret_cast<const float*>(xbase + (uint64_t)(cj[u] & kSweepColMask) * ldx_bytes), xs[u]);
        }
      } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
          for (int i = 0; i < VW; ++i) xs[u][i] = 0.f;
          if (live && base + j0 + u < len)
            load_vec<VW>(reinterpret_cast<const float*>(xbase + (uint64_t)(cj[u] & kSweepColMask) * ldx_bytes), xs[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int rid = (int)(cj[u] >> (32 - kSweepRowBits));
        if ((full || base + j0 + u < len) && rid != cur) {
          flush(cur);
          cur = rid;
        }
#pragma unroll
        for (int i = 0; i < VW; ++i) acc[i] = fmaf(vs[u], xs[u][i], acc[i]);
      }
    }
    cw = cw_next;
    v = v_next;
  }
  flush(cur);

  if (live) {
#pragma unroll 1
    for (int r = 0; r < R; ++r) {
      const int32_t row = slot_row[T * R + r];
      if (row < 0) continue;
      const int32_t so = slot_out[T * R + r];
      float out[VW];
#pragma unroll
      for (int i = 0; i < VW; ++i) out[i] = mine[r * kRowStride + i];
      if (so >= 0)
        store_out<VW>(partial + (int64_t)so * ldp + f0, nf, out, 0.f, MGGCN_EPI_NONE, false);
      else
        store_out<VW>(Y + (int64_t)row * ldy + f0, nf, out, beta, epi, true);
    }
  }
}

template <int LPR, int R>
int launch_lpr(const SweepSet& ss, const float* X, int64_t ldx, int F, int n_chunks, float beta, int epi,
               float* Y, int64_t ldy, float* partial, int64_t ldp, hipStream_t st) {
  constexpr int TPW = 64 / LPR;
  const int64_t teams_per_block = (kThreads / 64) * TPW;
  const int64_t blocks = (ss.n_teams / teams_per_block) * n_chunks;  // n_teams is padded to 256
  MGGCN_REQUIRE(blocks < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "SpMM grid of %lld blocks too large",
                (long long)blocks);
  spmm_sweep<4, LPR, R><<<(unsigned)blocks, kThreads, 0, st>>>(
      ss.d_team_begin, ss.d_scol, ss.d_sval, ss.d_slot_row, ss.d_slot_out, X, (uint32_t)(ldx * 4), F, n_chunks,
      beta, epi, Y, ldy, partial, ldp);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

template <int R>
int launch_r(const SweepSet& ss, const float* X, int64_t ldx, int F, int lpr, int n_chunks, float beta, int epi,
             float* Y, int64_t ldy, float* partial, int64_t ldp, hipStream_t st) {
  switch (lpr) {
    case 4: return launch_lpr<4, R>(ss, X, ldx, F, n_chunks, beta, epi, Y, ldy, partial, ldp, st);
    case 8: return launch_lpr<8, R>(ss, X, ldx, F, n_chunks, beta, epi, Y, ldy, partial, ldp, st);
    case 16: return launch_lpr<16, R>(ss, X, ldx, F, n_chunks, beta, epi, Y, ldy, partial, ldp, st);
    case 32: return launch_lpr<32, R>(ss, X, ldx, F, n_chunks, beta, epi, Y, ldy, partial, ldp, st);
    case 64: return launch_lpr<64, R>(ss, X, ldx, F, n_chunks, beta, epi, Y, ldy, partial, ldp, st);
    default: break;
  }
  return MGGCN_E_UNSUPPORTED;
}

}  // namespace

int launch_sweep(const SweepSet& ss, const float* X, int64_t ldx, int F, int lpr, int n_chunks, float beta,
                 int epi, float* Y, int64_t ldy, float* partial, int64_t ldp, void* stream) {
  hipStream_t st = as_stream(stream);
  switch (ss.R) {
    case 4: return launch_r<4>(ss, X, ldx, F, lpr, n_chunks, beta, epi, Y, ldy, partial, ldp, st);
    case 8: return launch_r<8>(ss, X, ldx, F, lpr, n_chunks, beta, epi, Y, ldy, partial, ldp, st);
    case 16: return launch_r<16>(ss, X, ldx, F, lpr, n_chunks, beta, epi, Y, ldy, partial, ldp, st);
    default: break;
  }
  return MGGCN_E_UNSUPPORTED;
}

}  // namespace mggcn
