// Host sanitizer job for the HIP library's host logic: the library is built with
// -fsanitize=address,undefined on the host side only (tests/test_sanitizers.py) and this driver
// sweeps seeded descriptors through everything that runs before a launch -- validation, workspace
// sizes, the split plans of the key and query walks, the projection and Linformer split counts --
// and through the row maps of the two ownerships.  No kernel is launched: every compute call is
// made with an argument that the host rejects.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "rsa.h"
#include "rsa_common.h"

static uint64_t state = 0x853C49E6748FEA9Bull;
static uint64_t next() { state ^= state >> 12; state ^= state << 25; state ^= state >> 27; return state * 0x2545F4914F6CDD1Dull; }
static int64_t pick(int64_t lo, int64_t hi) { return lo + (int64_t)(next() % (uint64_t)(hi - lo + 1)); }

static int check_row_map(const rsa_desc &d) {
  rsa::Dims dm{};
  dm.N = d.N; dm.rank_begin = d.rank_begin; dm.rank_end = d.rank_end; dm.L = d.L; dm.c = d.L / d.N;
  dm.Lq = (int64_t)(d.rank_end - d.rank_begin) * dm.c; dm.zigzag = (d.flags & RSA_OWN_ZIGZAG) ? 1 : 0;
  const rsa::RowMap m = rsa::make_row_map(dm);
  std::vector<char> seen((size_t)d.L, 0);
  for (int64_t r = 0; r < dm.Lq; ++r) {
    const int64_t g = m(r);
    if (g < 0 || g >= d.L || seen[(size_t)g]) return 1;          // a token is owned once
    seen[(size_t)g] = 1;
    const int owner = m.owner(g);
    if (owner != d.rank_begin + (int)(r / dm.c)) return 1;       // by the rank whose rows hold it
    if (m.key_of(owner, r % dm.c) != g) return 1;                // and key_of walks the same tokens
  }
  return 0;
}

int main() {
  int bad = 0;
  long valid = 0, invalid = 0;
  void *p = reinterpret_cast<void *>(0x1000);
  for (int it = 0; it < 20000; ++it) {
    rsa_desc d{};
    d.B = (int32_t)pick(0, 9); d.Z = (int32_t)pick(0, 17);
    d.A = (int32_t)(pick(0, 5) * 64 - (pick(0, 9) == 0 ? 32 : 0));
    d.N = (int32_t)pick(0, 40);
    const int64_t c = pick(0, 70) * 64 + (pick(0, 19) == 0 ? 32 : 0);
    d.L = (d.N > 0 ? d.N : 1) * c + (pick(0, 29) == 0 ? 1 : 0);
    d.rank_begin = (int32_t)pick(-1, d.N > 0 ? d.N - 1 : 0);
    d.rank_end = (int32_t)pick(d.rank_begin, d.N + 1);
    d.causal = (int32_t)pick(0, 1);
    d.dtype = (int32_t)pick(0, 2);
    d.scale = pick(0, 3) == 0 ? 0.0f : (float)pick(-1, 100) * 0.01f;
    d.flags = (uint32_t)pick(0, 9);
    if (pick(0, 3) == 0) {   // some strided layouts, some of them wrong
      const int64_t row = d.A + pick(-1, 3) * 8, head = row * pick(1, 3), batch = head * (d.Z > 0 ? d.Z : 1) * (c > 0 ? c : 1) * 40;
      int64_t *st = pick(0, 1) ? d.kv_stride : d.q_stride;
      st[0] = batch; st[1] = head; st[2] = row;
    }
    const size_t w0 = rsa_workspace_bytes(&d, 0), w1 = rsa_workspace_bytes(&d, 1);
    const size_t wp = rsa_proj_workspace_bytes(&d, (int32_t)(pick(0, 20) * 64));
    const size_t wl = rsa_linformer_workspace_bytes(&d, (int32_t)(pick(0, 8) * 64));
    (void)wp; (void)wl;
    // a null tensor pointer is refused after validation and before any launch
    const int rc = rsa_forward(&d, nullptr, p, p, p, static_cast<float *>(p), p, (size_t)1 << 40, nullptr);
    const int rb = rsa_backward(&d, nullptr, p, p, p, p, static_cast<float *>(p), p, p, p, p, (size_t)1 << 40, nullptr);
    if (rc == RSA_OK || rb == RSA_OK) bad = 1;
    if (rc == RSA_ERR_NULL) {          // the descriptor itself was valid
      ++valid;
      if (rb != RSA_ERR_NULL) bad = 1;
      if ((d.flags & RSA_MODE_STAGED) && (w0 == 0 || w1 == 0)) bad = 1;
      if (!(d.flags & RSA_MODE_STAGED) && w1 < 8u * (size_t)d.B * d.Z * (size_t)(d.rank_end - d.rank_begin) * (size_t)(d.L / d.N)) bad = 1;
      if (d.L <= 8192) bad |= check_row_map(d);
      // a workspace one byte short is refused on the host
      if (w1 > 0 && rsa_backward(&d, p, p, p, p, p, static_cast<float *>(p), p, p, p, p, w1 - 1, nullptr) != RSA_ERR_WORKSPACE) bad = 1;
      if (w0 > 0 && rsa_forward(&d, p, p, p, p, static_cast<float *>(p), p, w0 - 1, nullptr) != RSA_ERR_WORKSPACE) bad = 1;
    } else {
      ++invalid;
      if (w0 != 0 || w1 != 0) bad = 1;   // an invalid descriptor has no workspace size
    }
    if (bad) { std::fprintf(stderr, "descriptor %d failed\n", it); break; }
  }
  if (valid < 500 || invalid < 500) bad = 1;   // the sweep must reach both sides
  std::printf(bad ? "SANITIZE_HOST_FAILED\n" : "SANITIZE_HOST_OK valid=%ld invalid=%ld\n", valid, invalid);
  return bad;
}
