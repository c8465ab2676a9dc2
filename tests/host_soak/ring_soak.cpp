// CPU-only soak of the library's host state machine (descriptor validation and the closed-form
// ring tables of paper_2603_17051_amd/csrc/ring_state.hpp) against a naive ring written here:
// a list of slots, a new frame takes the lowest empty slot, else the slot of the oldest frame
// that is not a sink (Sec. 3.2: sinks are kept, the window slides).  Built by the test with
// -fsanitize=address,undefined; stops at the first mismatch with exit code 1.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../paper_2603_17051_amd/csrc/ring_state.hpp"

namespace {

struct Rng {  // xorshift64*, seeded
  uint64_t s;
  explicit Rng(uint64_t seed) : s(seed * 0x9E3779B97F4A7C15ull + 1) {}
  uint64_t next() {
    s ^= s >> 12; s ^= s << 25; s ^= s >> 27;
    return s * 0x2545F4914F6CDD1Dull;
  }
  int below(int n) { return (int)(next() % (uint64_t)n); }
};

struct NaiveRing {
  int C, S;
  int64_t start = 0, next_n = 0;
  std::vector<int64_t> slot;  // frame number held, -1 = empty
  NaiveRing(int c, int s) : C(c), S(s), slot(c, -1) {}
  void reset(int64_t st) { start = st; next_n = 0; std::fill(slot.begin(), slot.end(), -1); }
  int append_frame() {
    int at = -1;
    for (int i = 0; i < C && at < 0; ++i)
      if (slot[i] < 0) at = i;
    if (at < 0) {
      int64_t oldest = INT64_MAX;
      for (int i = 0; i < C; ++i)
        if (slot[i] >= S && slot[i] < oldest) { oldest = slot[i]; at = i; }
    }
    slot[at] = next_n++;
    return at;
  }
  int rank_of(int i) const {  // position of slot i's frame among the residents in stream order
    if (slot[i] < 0) return -1;
    int r = 0;
    for (int j = 0; j < C; ++j)
      if (slot[j] >= 0 && slot[j] < slot[i]) ++r;
    return r;
  }
};

int fail(const char* what, int C, int S, int Fc, long op, int b, int s, long got, long want) {
  std::printf("MISMATCH %s: C=%d S=%d Fc=%d op=%ld stream=%d slot=%d got=%ld want=%ld\n", what, C, S, Fc, op, b, s, got, want);
  return 1;
}

int soak(int C, int S, int Fc, int ops, uint64_t seed) {
  const int B = 3;
  astro_kvcache_desc_t d{};
  d.batch = B; d.heads = 2; d.head_dim = 64; d.grid_h = 2; d.grid_w = 3;
  d.capacity_frames = C; d.sink_frames = S; d.max_chunk_frames = Fc;
  d.rope_pairs_t = 12; d.rope_pairs_h = 10; d.rope_pairs_w = 10;
  d.dtype = ASTRO_BF16; d.flags = ASTRO_FLAG_HOST_ONLY; d.rope_base = 10000.0;
  astro::RingGeometry g{};
  if (astro::validate_desc(&d, &g) != ASTRO_OK) return fail("validate_desc", C, S, Fc, -1, 0, 0, 0, 0);
  astro::RingTables tables(B, C, S);
  std::vector<NaiveRing> naive(B, NaiveRing(C, S));
  Rng rng(seed);
  for (long op = 0; op < ops; ++op) {
    if (rng.below(10) == 0) {
      const int stream = rng.below(B + 1) - 1;  // -1 = all
      const int32_t st = rng.below(1000);
      tables.reset(stream, st);
      for (int b = 0; b < B; ++b)
        if (stream < 0 || stream == b) naive[b].reset(st);
    } else {
      const int n = 1 + rng.below(Fc);
      if (!tables.can_append(n)) return fail("can_append", C, S, Fc, op, 0, 0, 0, 1);
      for (int b = 0; b < B; ++b)
        for (int i = 0; i < n; ++i) {
          const int64_t number = naive[b].next_n;
          const int at = naive[b].append_frame();
          const int got = astro::slot_of_frame_number(number, C, S);
          if (got != at) return fail("slot_of_frame_number", C, S, Fc, op, b, at, got, at);
        }
      tables.append(n);
    }
    const std::vector<int32_t> sf = tables.slot_frame(), sr = tables.slot_rank();
    for (int b = 0; b < B; ++b) {
      if (tables.next_n(b) != naive[b].next_n) return fail("next_n", C, S, Fc, op, b, 0, tables.next_n(b), naive[b].next_n);
      int resident = 0;
      for (int s = 0; s < C; ++s) {
        const int64_t held = naive[b].slot[s];
        resident += held >= 0;
        const long want_frame = held < 0 ? -1 : (long)(naive[b].start + held);
        if (sf[(size_t)b * C + s] != want_frame) return fail("slot_frame", C, S, Fc, op, b, s, sf[(size_t)b * C + s], want_frame);
        if (sr[(size_t)b * C + s] != naive[b].rank_of(s)) return fail("slot_rank", C, S, Fc, op, b, s, sr[(size_t)b * C + s], naive[b].rank_of(s));
        const int64_t inv = astro::frame_number_in_slot(s, tables.next_n(b), C, S);
        if (inv != held) return fail("frame_number_in_slot", C, S, Fc, op, b, s, inv, held);
      }
      if (tables.resident(b) != resident) return fail("resident", C, S, Fc, op, b, 0, tables.resident(b), resident);
      const long evicted = naive[b].next_n - resident;
      if (tables.evicted(b) != evicted) return fail("evicted", C, S, Fc, op, b, 0, tables.evicted(b), evicted);
    }
  }
  return 0;
}

// random descriptors: validation must neither crash nor accept what breaks the tables' assumptions
int fuzz_descriptors(int n, uint64_t seed) {
  Rng rng(seed);
  auto pick = [&](int lo, int hi) { return lo + rng.below(hi - lo + 1); };
  for (int i = 0; i < n; ++i) {
    astro_kvcache_desc_t d{};
    d.batch = pick(-2, 70); d.heads = pick(-1, 40); d.head_dim = (rng.below(4) == 0) ? pick(0, 200) : (rng.below(2) ? 64 : 128);
    d.grid_h = pick(-1, 70); d.grid_w = pick(-1, 70);
    d.capacity_frames = pick(-1, 300); d.sink_frames = pick(-2, 300); d.max_chunk_frames = pick(-1, 300);
    if (rng.below(2)) { d.rope_pairs_t = d.head_dim / 2 - 2 * (d.head_dim / 6); d.rope_pairs_h = d.rope_pairs_w = d.head_dim / 6; }
    else { d.rope_pairs_t = pick(-2, 40); d.rope_pairs_h = pick(-2, 40); d.rope_pairs_w = pick(-2, 40); }
    d.dtype = pick(-1, 2); d.flags = pick(0, 16) | ASTRO_FLAG_HOST_ONLY; d.block_frames = pick(-2, 5);
    d.rope_base = rng.below(5) == 0 ? 0.5 : 10000.0;
    astro::RingGeometry g{};
    const int rc = astro::validate_desc(&d, &g);
    if (rc != ASTRO_OK) continue;
    const bool sane = g.B >= 1 && g.B <= ASTRO_MAX_BATCH && g.C >= 1 && g.S >= 0 && g.S < g.C && g.Lw == g.C - g.S &&
                      g.max_chunk >= 1 && g.max_chunk <= g.Lw && g.T == g.gh * g.gw && (g.D == 64 || g.D == 128) &&
                      (g.n_t + g.n_h + g.n_w == 0 || g.n_t + g.n_h + g.n_w == g.D / 2);
    if (!sane) {
      std::printf("validate_desc accepted an inconsistent descriptor (case %d)\n", i);
      return 1;
    }
    if (soak(g.C, g.S, g.max_chunk, 40, seed + i)) return 1;
  }
  return 0;
}

}  // namespace

int main(int argc, char** argv) {
  const int ops = argc > 1 ? std::atoi(argv[1]) : 10000;
  const int shapes[][3] = {{1, 0, 1}, {2, 1, 1}, {4, 0, 1}, {4, 1, 3}, {5, 4, 1}, {7, 2, 5}, {12, 1, 3}, {18, 0, 3},
                           {21, 3, 3}, {12, 11, 1}, {64, 5, 17}, {256, 3, 11}};
  long total = 0;
  for (const auto& sh : shapes) {
    if (soak(sh[0], sh[1], sh[2], ops, 20260317u + sh[0] * 1000 + sh[1] * 10 + sh[2])) return 1;
    total += ops;
  }
  if (fuzz_descriptors(4000, 77)) return 1;
  std::printf("ring soak ok: %ld random append/reset calls over %zu shapes, 4000 random descriptors\n", total,
              sizeof(shapes) / sizeof(shapes[0]));
  return 0;
}
