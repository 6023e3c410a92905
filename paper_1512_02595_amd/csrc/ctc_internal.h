// Internal interfaces between the host launcher and the HIP kernels of the CTC library.
// Not part of the public ABI (that is include/ctc_mi355x.h).
#pragma once

#include <cstddef>
#include <algorithm>
#include <cstdint>
#include <vector>

#include "ctc_mi355x.h"

#ifndef CTC_STREAMING_MB
#define CTC_STREAMING_MB 128
#endif

namespace ctc {

// Per-utterance record, identical on host and device (48 bytes).
struct Utt {
    int32_t Tb;        // frames of this utterance (input_lengths[b])
    int32_t L;         // label length
    int32_t lab_off;   // offset of its label string in the flat label array
    int32_t flags;     // bit 0: the lattice runs (Tb > 0 and an alignment exists);
                       // bit 1: lengths or labels failed the device-side checks (cost NaN)
    int32_t f_off;     // frames of all earlier utterances: offset of its blank emissions [Tb]
    int32_t waves;     // wavefronts its lattice chains use when a lane owns one state pair (log-domain
                       // chains, and linear-domain chains of at most 64 pairs)
    int32_t halo;      // lanes per wavefront that recompute the wavefront below (0: none)
    int32_t poll_budget; // LDS polls a wavefront of its chains may spend waiting on a neighbour before it gives up
    int64_t e_off;     // offset (floats) of its label emissions
    int64_t ab_off;    // offset (8-byte words) of its alpha/beta blocks [Tb][lattice_pitch(L)]
    int32_t e_pitch;   // row pitch (floats) of its emission block: L (a frame's gathered emissions, one
                       // per label position) or the frames of a symbol's row (symbol-major block)
    int32_t e_direct;  // layout of the emission block: kEmitGathered or kEmitSymbolMajor (emission_layout)
    int32_t waves2;    // the same plan for linear-domain chains of more than 64 pairs, whose lanes own
    int32_t halo2;     // two neighbouring pairs each (plan_waves2)
};
static_assert(sizeof(Utt) == 64, "Utt is copied word by word and read with scalar loads: keep it 8-byte sized");

// Alphabets up to this size skip the emission gather: a frame's normalised row is as small as
// the gathered emissions would be, and the rows themselves, transposed, are the emission block
// (emission_layout).
constexpr int kDirectMaxA = 64;
constexpr int kDeviceFoldMaxB = 512;  // device-resident metadata: utterances up to which the narrow softmax launch builds the records
constexpr int kNarrowMaxB = 128;      // utterances whose frame counts travel in the narrow softmax launch's arguments
constexpr int kFlagFrames = 64;       // frames per word of Layout::row_flags = frames per workgroup of the narrow softmax launch

#if defined(__HIPCC__)
#define CTC_HOST_DEVICE __host__ __device__
#else
#define CTC_HOST_DEVICE
#endif

constexpr int kChunkSteps = 8;        // = kChunk (below): steps between two possible hand-overs

// How the L+1 state pairs of a chain are spread over wavefronts.
struct WavePlan {
    int waves;
    int halo;
    bool barrier;      // too long for a halo: 64 pairs per wavefront, one barrier per step
};

// Wavefronts and halo width for a label of this length.  Measured on gfx950: with one
// wavefront per SIMD (up to 4) a step costs about 210 clocks and a hand-over about 500; with
// several per SIMD the vector ALU is the limit (about 170 clocks per wavefront-step) and part
// of a hand-over's latency hides behind the other wavefronts (about 350).
// (Host and device: the launcher plans on the host, the device-metadata entry point on the GPU.)
// `crowded`: the launch has more wavefronts than the chip runs side by side at one per SIMD, so
// what counts is the total work (wavefront-steps plus hand-overs), not one chain's latency.
CTC_HOST_DEVICE inline WavePlan plan_waves(int label_length, bool crowded = false)
{
    const int pairs = label_length + 1;
    if (pairs <= 64) return {1, 0, false};
    // Hand-overs happen on chunk boundaries: the halo is a multiple of kChunk (8 .. 32), and
    // the lanes handed up must themselves be exact ones (halo <= 64 - halo).
    WavePlan best{16, 0, true};
    float best_cost = 1e30f;
    const int w0 = (pairs - 8 + 55) / 56;       // fewest wavefronts with a halo of 8: w * 56 + 8 >= pairs
    for (int w = w0; w <= 16 && w <= w0 + 4; ++w) {
        // w * (64 - halo) + halo >= pairs
        int halo = (64 * w - pairs) / (w - 1);
        if (halo > 32) halo = 32;
        halo -= halo % 8;
        if (halo < 8) continue;
        const int per_simd = (w + 3) / 4;
        // the last term prefers fewer wavefronts when the estimates are close
        const float cost = crowded ? w * (170.0f + 350.0f / halo)
                                   : ((per_simd == 1) ? 210.0f + 500.0f / halo : per_simd * 170.0f + 350.0f / halo) + 4.0f * w;
        if (cost < best_cost) {
            best_cost = cost;
            best = {w, halo, false};
        }
    }
    return best;
}

// The same for chains whose lanes own two neighbouring state pairs each (linear domain, more than
// 64 pairs).  A wavefront then covers 128 pairs, an error at lane 0 needs two steps per lane to
// move up, so a halo of h lanes lasts 2h steps: h is a multiple of 4 (hand-overs on chunk
// boundaries), at most 16 (the exchange buffer).  Sixteen wavefronts hold any supported label.
// Measured on gfx950: about 150 clocks per step with one wavefront per SIMD, 600 per hand-over.
CTC_HOST_DEVICE inline WavePlan plan_waves2(int label_length, bool crowded = false)
{
    const int lanes = (label_length + 2) / 2;          // ceil((L + 1) / 2)
    if (lanes <= 64) return {1, 0, false};
    WavePlan best{16, 4, false};
    float best_cost = 1e30f;
    // Fewest wavefronts with a halo of 4: w * 60 + 4 >= lanes.  The halo reaches its cap of 16 within
    // three more wavefronts (lanes / 48 against lanes / 60, lanes <= 512), and beyond that a further
    // wavefront only costs: no need to look further (the device-side planners run this per utterance).
    const int w_first = (lanes - 4 + 59) / 60 > 2 ? (lanes - 4 + 59) / 60 : 2;
    for (int w = w_first; w <= 16 && w <= w_first + 3; ++w) {
        // w * (64 - halo) + halo >= lanes
        int halo = (64 * w - lanes) / (w - 1);
        if (halo > 16) halo = 16;
        halo -= halo % 4;
        if (halo < 4) continue;
        const int per_simd = (w + 3) / 4;
        const float cost = crowded ? w * (110.0f + 300.0f / halo)
                                   : ((per_simd == 1) ? 150.0f : per_simd * 110.0f) + 300.0f / halo + 4.0f * w;
        if (cost < best_cost) {
            best_cost = cost;
            best = {w, halo, false};
        }
    }
    return best;
}

// Which of the two plans a linear-domain chain uses.  Measured on gfx950: a step of a two-pair
// lane takes about 180 clocks against 120 for a one-pair lane, and a hand-over 560, so while a
// label's one-pair plan keeps to one wavefront per SIMD (at most 4) it is the faster one; beyond
// that, and in crowded launches, where wavefront-steps count and not one chain's latency, the
// two-pair plan with half the wavefronts wins.  Where the emission block is symbol-major
// (emission_layout) a two-pair lane's fetches are cheap, and the two-pair plan also wins against
// a one-pair plan that hands over every chunk (halo 8): 64 utterances of 600 frames, lattice
// launch for labels of 215 symbols 52.1 -> 46.5 us, of 230 symbols 52.9 -> 50.1 us; up to 207
// symbols (halo 16 or more) the one-pair plan stays ahead by up to 4 us.
CTC_HOST_DEVICE inline bool two_pairs_per_lane(int label_length, bool crowded, bool symbol_major = false)
{
    if (label_length + 1 <= 64) return false;
    const WavePlan one = plan_waves(label_length, crowded);
    return crowded || one.barrier || one.waves > 4 || (symbol_major && one.halo < 2 * kChunkSteps);
}

// The plans of every label length, packed: what a launch that builds its utterance records on the
// GPU carries in its arguments instead of evaluating plan_waves per utterance there.
//   one[L]: bits 0..3 wavefronts - 1, bits 4..6 halo / 8 (plan_waves), bit 7 two_pairs_per_lane
//   two[L]: bits 0..3 wavefronts - 1, bits 4..6 halo / 4 (plan_waves2)
struct PlanTable {
    uint8_t one[CTC_MAX_LABEL_LENGTH + 1];
    uint8_t two[CTC_MAX_LABEL_LENGTH + 1];
    CTC_HOST_DEVICE int waves1(int L) const { return (one[L] & 15) + 1; }
    CTC_HOST_DEVICE int halo1(int L) const { return ((one[L] >> 4) & 7) * 8; }
    CTC_HOST_DEVICE bool two_pairs(int L) const { return (one[L] & 128) != 0; }
    CTC_HOST_DEVICE int waves2(int L) const { return (two[L] & 15) + 1; }
    CTC_HOST_DEVICE int halo2(int L) const { return (two[L] >> 4) * 4; }
};
// For labels up to max_label (kept per distinct request: a training run asks for one or two).
const PlanTable& plan_table(int max_label, bool crowded, bool symbol_major);

// How a launch's label emissions are laid out (Utt::e_direct).
//   kEmitGathered:    [frame][label position], L floats per frame (alphabets above kDirectMaxA)
//   kEmitSymbolMajor: [symbol][frame]: the normalised rows themselves, transposed, so that a
//                     symbol's frames lie side by side and a lane fetches the frames of a chunk
//                     in two 16-byte loads instead of eight loads a row apart
// Measured on gfx950 against the rows as they are ([frame][symbol]): English minibatch, lattice
// launch 60.4 -> 58.4 us; long utterances (two wavefronts of a chain on one SIMD, instruction
// issue the limit) 203 -> 168 us.
constexpr int kEmitGathered = 0, kEmitSymbolMajor = 1;
CTC_HOST_DEVICE inline int emission_layout(int A) { return A <= kDirectMaxA ? kEmitSymbolMajor : kEmitGathered; }

// The sink of a lattice launch: for each of its up to 2 B chain workgroups, kSinkBytes for each of the
// up to kSinkWaves wavefronts.
constexpr int kSinkWaves = 16, kSinkBytes = 64;

constexpr int kUttRuns = 1;
constexpr int kUttInvalid = 2;
// Set by the softmax launch when some emission of the utterance is too improbable for the
// linear-domain recursion (below 2^kLinearMinLog2): its chains then run in the log domain.
// (Also set for every utterance of a launch that uses the one-barrier-per-step kernel.)
constexpr int kUttLogDomain = 4;
// Linear-domain chains of this utterance give two neighbouring state pairs to every lane
// (plan_waves2) instead of one (plan_waves): see two_pairs_per_lane.
constexpr int kUttTwoPairs = 8;
// Overlapped launches (kTaskRows): the utterance's gradient rows are written by the gradient launch,
// not by the lattice launch's workers.
constexpr int kUttGradientLater = 16;
constexpr float kLinearMinLog2 = -100.0f;
// Utterances of more frames than this run the log domain whatever their emissions: the lanes'
// exponents, which fall by up to 100 per frame, must stay clear of kNoExponent and of int32's end.
constexpr int kLinearMaxFrames = 1 << 21;
// Utterances with fewer than this many frames to spare (frames - symbols - repeated neighbours) run the log
// domain too.  Where hardly a frame is to spare the alignments run along the front of the lattice, and the
// states behind the front, whose mass can no longer reach the end, may outweigh it by more than the lanes'
// frames of the linear domain hold (lane_frame in the kernels: 2^950 within ten state pairs); with this
// many frames to spare every state that near the front can still reach the end.  Measured before the rule:
// 138 frames, 91 symbols, 47 repeats, emissions down to 2^-95: the front 2^1900 below its neighbours, the
// linear domain's cost +inf.
constexpr int kTightFrames = 16;
CTC_HOST_DEVICE inline bool tight_fit(int frames, int label_length, int repeats)
{
    return frames - label_length - repeats < kTightFrames;
}
// Lattice wavefronts of one launch beyond which chains are planned for total work: two per SIMD
// of the 256 compute units.
constexpr int kCrowdedWaves = 2 * 4 * 256;
// The order in which the lattice launch takes its chains (entry = utterance * 2 + direction).
// `utt`: the utterances whose lattice runs, heaviest (frames x wavefronts) first; `dirs`: 2 when
// the backward chains run too.  Up to `n_cu` chains (one per compute unit) keep that order.
// Beyond that, chains share compute units, and the launch lasts as long as the busiest SIMD:
// a chain's wavefront nearly fills the SIMD it runs on, so two on one SIMD take the sum of
// their times.  The workgroup dispatcher, as observed on gfx950, hands workgroup i to compute
// unit i mod n_cu and, on a compute unit, starts each further workgroup one SIMD later than
// the one before it.  The order is therefore built in rounds of n_cu workgroups that follow
// the SIMDs' loads under that model: a round whose wavefronts land on SIMDs busier than the
// compute units' average takes the lightest chains left, any other the heaviest, and within
// a round the lightest chain goes to the compute unit whose landing SIMD is the busiest.
// (Should the dispatcher place workgroups otherwise, the order is merely not the best one.)
constexpr int kXcds = 8;     // accelerator dies of an MI355X, each with its own L2
constexpr int kChainBlock = 2 * kXcds;

inline void order_chains(const int32_t* utt, const int32_t* frames, const int32_t* waves, int n, int dirs,
                         int n_cu, int32_t* order)
{
    struct Chain { int32_t entry, frames, waves; };
    const int total = n * dirs;
    std::vector<Chain> chains(static_cast<size_t>(total));
    // Workgroup i runs on die (XCD) i mod kXcds.  The two chains of an utterance read the same
    // emissions; kChainBlock forward chains followed by the backward chains of the same
    // utterances puts the two a multiple of kXcds entries apart, on one die and its L2.
    for (int i0 = 0, at = 0; i0 < n; i0 += kChainBlock)
        for (int d = 0; d < dirs; ++d)
            for (int i = i0; i < std::min(n, i0 + kChainBlock); ++i) chains[at++] = {utt[i] * 2 + d, frames[i], waves[i]};
    if (n_cu < 1 || total <= n_cu) {
        for (int i = 0; i < total; ++i) order[i] = chains[i].entry;
        return;
    }
    std::vector<int64_t> load(static_cast<size_t>(n_cu) * 4, 0);
    std::vector<int> cus(static_cast<size_t>(n_cu));
    int lo = 0, hi = total, pos = 0;
    for (int round = 0; lo < hi; ++round) {
        const int k = std::min(n_cu, hi - lo), s = round & 3;
        int64_t landing = 0, all = 0, least = INT64_MAX, most = 0;
        for (int c = 0; c < k; ++c) {
            const int64_t l = load[static_cast<size_t>(c) * 4 + s];
            landing += l;
            least = std::min(least, l);
            most = std::max(most, l);
            for (int q = 0; q < 4; ++q) all += load[static_cast<size_t>(c) * 4 + q];
        }
        const bool lightest = landing * 4 > all;
        const int first = lightest ? hi - k : lo;      // chains[first .. first + k): heaviest first
        if (lightest) hi -= k; else lo += k;
        for (int c = 0; c < k; ++c) cus[c] = c;
        if (least != most)                              // busiest landing SIMD first; it gets the lightest chain
            std::stable_sort(cus.begin(), cus.begin() + k, [&](int a, int b) {
                return load[static_cast<size_t>(a) * 4 + s] > load[static_cast<size_t>(b) * 4 + s];
            });
        for (int j = 0; j < k; ++j) {
            const Chain& ch = (least != most) ? chains[first + k - 1 - j] : chains[first + j];
            const int c = cus[j];
            order[pos + c] = ch.entry;
            for (int w = 0; w < ch.waves; ++w) load[static_cast<size_t>(c) * 4 + ((s + w) & 3)] += ch.frames;
        }
        pos += k;
    }
}

// Lattice size (alpha and beta together) beyond which the gradient kernel reads it with loads
// that leave no copy in the caches.  Measured on gfx950: 0.4 GB (512 utterances) 141 -> 104 us with
// such loads, 53 MB (64 utterances) 14.9 -> 15.7 us.
constexpr size_t kStreamingLatticeBytes = size_t(CTC_STREAMING_MB) << 20;

// Gradient rows inside the lattice launch.  A launch with fewer chains than compute units leaves
// the rest of the chip idle for as long as the longest chain runs, while the gradient of an
// utterance could start the moment both of its chains have ended.  Such launches therefore carry
// extra workgroups after the chains' ("workers") whose wavefronts share out a list of tasks: a task
// is kTaskRows consecutive frames of one utterance.  The list holds first the tasks that need no
// lattice (zero fill of padding frames and of utterances without an alignment), then the frames
// of the utterances in the order in which their chains are expected to end; a wavefront whose
// next task belongs to an utterance whose chains are still running waits for that utterance's
// counter (bounded polling).  Chains are launched first, so they are resident before any worker:
// a worker only ever waits for work that is running.
// A worker reads an utterance's lattice out of the L2 of the die (XCD) that its chains ran on, so
// the list has a section per die, for the workers of that die.
// The list as the host prepares it (part of the metadata image): `entries` runs of tasks,
//   die[d]      first entry of die d's section (die[kXcds] = entries)
//   prefix[e]   number of tasks before entry e (prefix[entries] = all tasks)
//   info[e]     utterance (low 16 bits); log2 of the rows per task; kTaskWaits if its chains must have ended
//   first[e]    first block (of that many rows) of the run
constexpr int kTaskRowsLog2 = 3, kTaskRows = 1 << kTaskRowsLog2;
constexpr int kWorkerSharePercent = 80;     // utterances whose chains end in the last fifth of the launch are left to the gradient launch
constexpr int kTaskRowsShift = 16;
constexpr int kTaskWaits = 1 << 30;
constexpr int kMaxTaskEntries = 256;        // two runs per utterance: overlapped launches have at most 128 utterances
constexpr int kWorkerWavesPerCu = 16;       // worker wavefronts per idle compute unit (the chains' register budget allows 4 per SIMD)
constexpr int kDoneStride = 64;             // ints between two utterances' counters: each in a 256-byte block of its own, so that
                                            // the waiting for one utterance does not hit the memory channel of the others
constexpr int kWherePolls = 256;            // polls before a worker stops asking where an utterance's chains run (they start within microseconds)
constexpr int kWorkerPollBudget = 1 << 22;  // polls (each followed by a short sleep) before a worker gives an utterance up
constexpr int kDefaultPollBudget = 1 << 22;   // enough for seconds of waiting: only a stuck neighbour exhausts it
constexpr int kMaxBatch = 65535;         // utterances index the second grid dimension of the row kernels
constexpr int kMaxDeviceMetaB = 4096;   // utterances the device-side planner ranks in LDS

// The lattice kernel reads emissions ahead of the recursion without bounds checks.  It
// fetches kChunk steps at a time and, at the start of a pass that begins at step s0 <= Tb-1,
// has requested steps up to s0 + 3*kChunk - 1 (two register sets, chain_schedule; with three sets,
// chain_schedule3, requests run up to 5 chunks ahead but a round's later ones only go out while a
// chunk of the chain is still to come, which bounds them the same): at most 3*kChunk - 1 rows past either end of
// an utterance's block (past the end going forward, before the start going backward).  These
// margins keep such reads inside the workspace; the values read there are never used.
constexpr int kChunk = kChunkSteps;   // steps whose emissions are fetched together (plan_waves: halo % 8 == 0)
constexpr int kOverFetchRows = 3 * kChunk;
constexpr int kBlankSlack = kOverFetchRows + kChunk;                          // floats, each side
constexpr int kLabelSlack = kOverFetchRows * (CTC_MAX_LABEL_LENGTH + 1);      // floats, each side

// Constants that lanes without a label state read as their emission, at the start of the
// label-emission region (inside its front slack): 20 floats of probability 0, then 20 of log 0.  Such
// a lane points at entry 8 of its 20: a fetch reads the 8 floats before it or the 8 after it, the
// first step the entry itself.
constexpr int kEmissionConstantRun = 20;
constexpr int kZeroEmission = 8, kLogZeroEmission = kEmissionConstantRun + 8, kEmissionConstants = 2 * kEmissionConstantRun;
static_assert(kChunk <= 8 && kEmissionConstants <= kLabelSlack, "constants sit inside the front slack");

// ---- where and when a chain reads its emissions -------------------------------------------------
// Shared by the lattice kernels and by the host-side replay that checks every read against the
// regions' bounds (ctc_debug_replay_emission_fetches): the kernels fetch ahead without bounds
// checks, so what they may touch is defined here, once.  Offsets are in floats from the start of
// the region (Layout::emit_label, Layout::emit_blank).

// Pointer of a lane's label emissions before step 0: at the emission of its label state in frame
// f0 (the chain's first frame), or at `constant` for a lane without a label state.  `symbol` is the
// state's symbol (symbol-major blocks: a row per symbol), `li` its label position (gathered blocks).
CTC_HOST_DEVICE inline int64_t label_emission_offset(const Utt& m, bool has_label, bool symbol_major, int symbol,
                                                     int li, int f0, int constant)
{
    if (!has_label) return constant;
    return kLabelSlack + m.e_off + (symbol_major ? static_cast<int64_t>(symbol) * m.e_pitch + f0
                                                 : static_cast<int64_t>(f0) * m.e_pitch + li);
}
// The same pointer moves by this much per step (gathered blocks: one row; symbol-major: one float),
// in the chain's direction fdir = +1 / -1; a lane without a label state stays where it is.
CTC_HOST_DEVICE inline int64_t label_emission_step(const Utt& m, bool has_label, bool symbol_major, int fdir)
{
    return !has_label ? 0 : (symbol_major ? fdir : static_cast<int64_t>(fdir) * m.e_pitch);
}
// Pointer of a lane's blank emissions: lane i of a chunk's load takes the frame of step (chunk start + i % kChunk).
CTC_HOST_DEVICE inline int64_t blank_emission_offset(const Utt& m, int f0, int fdir, int lane)
{
    return kBlankSlack + m.f_off + f0 + fdir * (lane & (kChunk - 1));
}
// The linear-domain chains take the blank's probability as an fp64 scalar, a chunk's kChunk frames in one
// scalar load out of a block of doubles (Layout::emit_blank64, same slack in doubles): the window of the
// chunk that starts at step s0 is w[0] .. w[kChunk - 1] from this offset, in frame order (a backward chain
// uses it last to first).
CTC_HOST_DEVICE inline int64_t blank64_window(const Utt& m, int f0, int fdir, int s0)
{
    return kBlankSlack + m.f_off + f0 + (fdir > 0 ? s0 : -s0 - (kChunk - 1));
}
// One fetch out of a symbol-major block reads the kChunk floats next to the pointer p in the chain's
// direction, p[first] .. p[first + kChunk - 1], and moves p on by kChunk steps.
CTC_HOST_DEVICE constexpr int fetch_window_first(bool backward) { return backward ? -kChunk : 1; }

// The order in which a chain requests (fetch) and consumes (run) the emissions of its steps
// 1 .. Tb-1, kChunk steps at a time, in two register sets a and b; each callback gets the first
// step of its chunk.  Step 0 is read directly before this.  The last requests reach up to
// 3 * kChunk - 1 steps beyond the chain's end: what kOverFetchRows provides for.
template <typename FetchA, typename FetchB, typename RunA, typename RunB, typename EndChunk>
CTC_HOST_DEVICE inline void chain_schedule(int Tb, FetchA&& fetch_a, FetchB&& fetch_b, RunA&& run_a, RunB&& run_b,
                                           EndChunk&& end_chunk)
{
    fetch_a(1);
    int s0 = 1;
    // Two whole chunks per round, with no branch on the step number inside: the compiler's count of the
    // memory operations in flight stays exact there, and a wavefront waits for the emissions it is
    // about to use only, not for the stores of the chunk before.
    for (; s0 + 2 * kChunk <= Tb; s0 += 2 * kChunk) {
        fetch_b(s0 + kChunk);
        run_a(s0, true);
        end_chunk();
        fetch_a(s0 + 2 * kChunk);
        run_b(s0 + kChunk, true);
        end_chunk();
    }
    // the last, short round (run_x(s0, false) checks every step against the end)
    if (s0 < Tb) {
        fetch_b(s0 + kChunk);
        run_a(s0, false);
        end_chunk();
        fetch_a(s0 + 2 * kChunk);
        if (s0 + kChunk < Tb) {
            run_b(s0 + kChunk, false);
            end_chunk();
        }
    }
}

// The same with three register sets a, b, c: a chunk's emissions are requested two chunks before they are
// used (a request out of the die's L2 takes longer than the 300 ns of a chunk).  The last requests reach up
// to 3 * kChunk - 1 steps beyond the chain's end, as with two sets.
template <typename FetchA, typename FetchB, typename FetchC, typename RunA, typename RunB, typename RunC, typename EndChunk>
CTC_HOST_DEVICE inline void chain_schedule3(int Tb, FetchA&& fetch_a, FetchB&& fetch_b, FetchC&& fetch_c, RunA&& run_a,
                                            RunB&& run_b, RunC&& run_c, EndChunk&& end_chunk)
{
    fetch_a(1);
    fetch_b(1 + kChunk);
    int s0 = 1;
    for (; s0 + 3 * kChunk <= Tb; s0 += 3 * kChunk) {       // three whole chunks per round (see chain_schedule)
        fetch_c(s0 + 2 * kChunk);
        run_a(s0, true);
        end_chunk();
        fetch_a(s0 + 3 * kChunk);
        run_b(s0 + kChunk, true);
        end_chunk();
        fetch_b(s0 + 4 * kChunk);
        run_c(s0 + 2 * kChunk, true);
        end_chunk();
    }
    if (s0 < Tb) {
        fetch_c(s0 + 2 * kChunk);
        run_a(s0, false);
        end_chunk();
        if (s0 + kChunk < Tb) {
            fetch_a(s0 + 3 * kChunk);
            run_b(s0 + kChunk, false);
            end_chunk();
            if (s0 + 2 * kChunk < Tb) {
                fetch_b(s0 + 4 * kChunk);
                run_c(s0 + 2 * kChunk, false);
                end_chunk();
            }
        }
    }
}

// With three register sets the blank's scalar window (blank64_window) goes out one chunk ahead only, together
// with the label emissions of the chunk after it: the chunk whose window accompanies the request for s0.
CTC_HOST_DEVICE inline int blank64_chunk_with(int s0) { return s0 - kChunkSteps > 1 ? s0 - kChunkSteps : 1; }

// Row pitch (8-byte words) of an utterance's lattice blocks: column 1 + i holds label state i.
CTC_HOST_DEVICE inline int64_t lattice_pitch(int64_t L) { return L + 2; }

// Byte offsets of the workspace regions, all multiples of 256.
struct Layout {
    size_t meta = 0;      // Utt[B]
    size_t order = 0;     // int32[2B]    the lattice launch's chains, one per workgroup: utterance * 2 + direction
                          //              (0 forward, 1 backward), -1 for a workgroup without one (order_chains)
    size_t labels = 0;    // int32[sumL]
    size_t tasks = 0;     // int32[9 + 3 * 2B + 1]  the workers' tasks: die[9], prefix[2B + 1], info[2B], first[2B] (see kTaskRows)
    size_t labels8 = 0;   // uint8[sumL]  the label strings once more, a byte per symbol (image only; narrow alphabets)
    size_t links = 0;     // int32[sumL]  grouping of the label positions by symbol (slot, count, first)
    size_t logp = 0;      // double[B]    log2 of the alignment mass
    size_t sink = 0;      // what lanes with nothing to store scribble on: kSinkBytes per wavefront of a lattice launch
    size_t chain_err = 0; // int32[B]     set when a lattice wavefront gave up waiting for its neighbour
    size_t done = 0;      // int32[B * kDoneStride]  wavefronts of the utterance's chains that have ended (overlapped launches)
    size_t domain = 0;    // int32[2 B]   per utterance and direction, nonzero: that chain ran in the log domain (published by
                          //              the chain for the gradient, which must know where its exponent rows are)
    size_t row_flags = 0; // int32[B * ceil(T / 64)]  narrow alphabets: per 64 frames of an utterance, nonzero if one of
                          //              their emissions is too small for the linear domain (written by the softmax
                          //              launch, one word per workgroup, so that nothing needs clearing beforehand)
    size_t status = 0;    // int32[B]     device-resident metadata, records built by the narrow softmax launch: nonzero
                          //              if the utterance's lengths or labels are invalid
    size_t where = 0;     // int32[2B]    1 + the die each chain's workgroup runs on
    size_t leftover = 0;  // int32[B]     utterances whose rows a worker had to leave to the gradient launch
    size_t lse = 0;       // float[B*T]   row-wise log2-sum-exp2 of the scaled logits
    size_t emit_blank = 0; // float[slack + sum Tb + slack]  emission of blank per frame: the probability y, or
                           // log2 y (negative) where y < 2^kLinearMinLog2 (plain log2 y in launches for
                           // the most probable alignment)
    size_t emit_blank64 = 0; // double[slack + sum Tb + slack]  the blank's probability once more, for the scalar loads of
                             // the linear-domain chains (blank64_window)
    size_t emit_label = 0; // float[slack + sum Tb*L + slack]  emission of each label position, same coding
                           // (sum Tb*A for small alphabets: emission_layout); the front slack starts with
                           // the constants that lanes without a label state read: probability 0 and log 0
    size_t alpha = 0;     // 8-byte words [sum Tb*(L+2)]: label states only, one unused column on either side
    size_t beta = 0;      // of a frame's row (lattice_pitch), so that a lane may store two neighbours at once
    size_t total = 0;
    size_t upload_bytes = 0;   // meta..labels are contiguous: the image the host prepares per call
    int64_t sumL = 0;
    int64_t frames = 0;
    int64_t emit_floats = 0;
    int64_t ab_doubles = 0;
};

// Fills `lay` from the batch shape. Returns a status (argument checks on sizes and lengths).
ctc_status_t make_layout(int T, int B, int A, const int32_t* label_lengths,
                         const int32_t* input_lengths, ctc_dtype_t dtype, Layout* lay);

// What a call computes, and so what its chains are run for:
//   kGrad  sum over alignments, label states of every frame stored (cost and gradient)
//   kLoss  sum over alignments, nothing stored (cost only; forward chain only)
//   kBest  maximum over alignments, one byte of predecessor choices stored per state pair and
//          frame (most probable alignment; forward chain only)
enum class Mode { kGrad, kLoss, kBest };

// The same for the device-metadata entry point: sized for B utterances of T frames and
// max_label symbols each.
ctc_status_t make_layout_bounds(int T, int B, int A, int max_label, ctc_dtype_t dtype, Layout* lay);

// Kernel launch parameters shared by all stages.
struct Launch {
    Mode mode;
    int T, B, A, blank;
    ctc_dtype_t dtype;
    int n_run;          // utterances whose lattice runs
    int n_chains;       // workgroups of the lattice launch (entries of the order array)
    int max_waves;      // wavefronts per lattice block
    int max_frames;     // longest utterance among those whose lattice runs
    int max_label;      // longest label of the batch
    bool needs_barrier; // some utterance's label leaves no room for a halo
    const void* x;
    void* grads;        // nullptr unless mode == kGrad
    int32_t* alignment; // [B][T], mode == kBest only
    float* costs;
    char* ws;           // workspace base
    const int32_t* labels;    // device: the label strings, addressed by Utt::lab_off (inside the workspace
                              // for the host-metadata entry points, the caller's array otherwise)
    const void* host_image;   // pinned host copy of the meta/order/labels regions (device-readable)
    int* host_flag;           // pinned host word the device sets to host_flag_value when the image is free;
                              // nullptr when there is no image
    int host_flag_value;
    // device-metadata entry point only
    const int32_t* dev_label_lengths;
    const int32_t* dev_input_lengths;
    int32_t* dev_status;
    int poll_budget;          // copied into every Utt record
    bool crowded;             // plan the chains for total work rather than latency (device planner)
    // Gradient rows inside the lattice launch (kTaskRows): 0 tasks = a gradient launch of its own.
    int n_tasks;
    int n_task_entries;
    int n_cu;                 // compute units of the device
    // Narrow alphabets, host metadata: there is no upload launch; the softmax launch reads the pinned image
    // itself and copies it into the workspace for the launches after it, and the lattice launch releases it.
    bool folded;
    // Device-resident metadata with workers: the softmax launch builds their task list (build_task_table) from the
    // lengths on the GPU; n_tasks and n_task_entries are then upper bounds, the list itself says how many there are.
    bool sequential_chains = false;   // measurements: forward and backward chains in two launches, one after the other
    bool device_tasks = false;
    int share_percent = 0;    // (kWorkerSharePercent, or what ctc_debug_set_overlap asked for)
    Layout lay;
};

// Each returns a hipError_t as int (0 = success). `stream` is a hipStream_t.
int launch_setup(const Launch& p, void* stream);       // host metadata: copies the image
int launch_plan(const Launch& p, void* stream);        // device metadata: builds meta and order on the GPU
int launch_softmax(const Launch& p, void* stream);
int launch_lattice(const Launch& p, void* stream);
int launch_gradient(const Launch& p, void* stream);   // kGrad
int launch_backtrace(const Launch& p, void* stream);   // kBest

}  // namespace ctc
