// CPU-only harness for the library's host code (geometry, validation, packer, unpacker) under
// AddressSanitizer and UndefinedBehaviorSanitizer.  Built by tests/test_host_sanitizers.py from
// csrc/owq_pack.cpp with g++ -fsanitize=address,undefined; reads a manifest of cases written by
// that test (layers, expected blobs from the CPU oracle's format code, expected status codes) and
// drives every one through the C entry points with buffers of exactly the stated sizes, so that
// any read or write past them is caught.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <sstream>
#include <string>
#include <vector>

#include "owq.h"

static std::vector<uint8_t> slurp(const std::string &path) {
  std::ifstream f(path, std::ios::binary);
  return std::vector<uint8_t>((std::istreambuf_iterator<char>(f)), std::istreambuf_iterator<char>());
}

int main(int argc, char **argv) {
  if (argc != 2) return 2;
  const std::string dir = argv[1];
  std::ifstream man(dir + "/manifest.txt");
  std::string line;
  int n_cases = 0;
  while (std::getline(man, line)) {
    if (line.empty()) continue;
    std::istringstream is(line);
    std::string name;
    int d_out, d_in, bits, gs, k, layout, null_mask, want;
    is >> name >> d_out >> d_in >> bits >> gs >> k >> layout >> null_mask >> want;
    // exact-size heap copies of every array (empty files give empty vectors: data() may be null)
    std::vector<uint8_t> codes = slurp(dir + "/" + name + ".codes"), scale = slurp(dir + "/" + name + ".scale"),
                         zero = slurp(dir + "/" + name + ".zero"), idx = slurp(dir + "/" + name + ".idx"),
                         ww = slurp(dir + "/" + name + ".ww"), blob = slurp(dir + "/" + name + ".blob"),
                         canon = slurp(dir + "/" + name + ".canon");
    owq_layer_desc_t d;
    d.d_out = d_out; d.d_in = d_in; d.bits = bits; d.group_size = gs; d.k = k; d.layout = layout;
    d.codes = (null_mask & 1) ? nullptr : codes.data();
    d.scale = (null_mask & 2) ? nullptr : reinterpret_cast<const uint16_t *>(scale.data());
    d.zero = (null_mask & 4) ? nullptr : reinterpret_cast<const uint16_t *>(zero.data());
    d.weak_idx = (null_mask & 8) ? nullptr : reinterpret_cast<const int32_t *>(idx.data());
    d.weak_w = (null_mask & 16) ? nullptr : reinterpret_cast<const uint16_t *>(ww.data());
    size_t bytes = 0;
    const owq_status_t sb = owq_packed_bytes(&d, &bytes);
    owq_layer_info_t info;
    const owq_status_t sg = owq_geometry(&d, &info);
    if (sb != sg) { std::printf("%s: owq_packed_bytes %d but owq_geometry %d\n", name.c_str(), sb, sg); return 1; }
    if (sb != OWQ_OK) {
      // a bad shape: the packer must say the same, and must not touch the buffer
      uint8_t guard[16];
      const owq_status_t sp = owq_pack_host(&d, guard, sizeof(guard));
      if ((int)sp != want || (int)sb != want) { std::printf("%s: status %d / %d, expected %d\n", name.c_str(), sb, sp, want); return 1; }
      ++n_cases;
      continue;
    }
    std::vector<uint8_t> out(bytes, 0xA5);
    const owq_status_t sp = owq_pack_host(&d, out.data(), out.size());
    if ((int)sp != want) { std::printf("%s: owq_pack_host %d, expected %d\n", name.c_str(), sp, want); return 1; }
    if (sp == OWQ_OK) {
      // the oracle's blob is the format proper; the tile layout's blob goes on with working memory, all zero
      const bool longer = layout == OWQ_LAYOUT_TILE && blob.size() == info.off_scratch && bytes >= blob.size();
      if ((bytes != blob.size() && !longer) || std::memcmp(out.data(), blob.data(), blob.size()) != 0) {
        std::printf("%s: packed bytes differ from the oracle's (%zu vs %zu bytes)\n", name.c_str(), bytes, blob.size());
        return 1;
      }
      for (size_t i = blob.size(); i < bytes; ++i)
        if (out[i] != 0) { std::printf("%s: working memory of a fresh blob is not zero\n", name.c_str()); return 1; }
      std::vector<uint8_t> back((size_t)d_out * d_in, 0xA5);
      if (owq_unpack_codes(out.data(), &info, back.data()) != OWQ_OK || back != canon) {
        std::printf("%s: unpacked codes differ\n", name.c_str());
        return 1;
      }
      // one byte too few must be refused, and nothing written
      if (bytes > 0) {
        std::vector<uint8_t> small(bytes - 1, 0x5A);
        if (owq_pack_host(&d, small.data(), small.size()) != OWQ_ERR_BUFFER) { std::printf("%s: short buffer accepted\n", name.c_str()); return 1; }
        for (uint8_t b : small) if (b != 0x5A) { std::printf("%s: short buffer written to\n", name.c_str()); return 1; }
      }
    }
    ++n_cases;
  }
  // null arguments
  size_t n = 0;
  owq_layer_info_t info;
  if (owq_packed_bytes(nullptr, &n) != OWQ_ERR_NULL || owq_geometry(nullptr, &info) != OWQ_ERR_NULL ||
      owq_pack_host(nullptr, &n, 8) != OWQ_ERR_NULL || owq_unpack_codes(nullptr, &info, nullptr) != OWQ_ERR_NULL) {
    std::printf("null arguments not refused\n");
    return 1;
  }
  std::printf("ok %d cases\n", n_cases);
  return 0;
}
