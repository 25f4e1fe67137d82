// Host-only driver of the graph packer for the sanitizer test: reads the caller-side
// arrays from binary files in the directory given as argv[1] and packs them.
#include <cstdio>
#include <string>
#include <vector>

#include "../paper_1711_01912_amd/csrc/cpeval_internal.hpp"

template <typename T>
static std::vector<T> read_all(const std::string &dir, const char *name) {
    std::vector<T> v;
    FILE *f = std::fopen((dir + "/" + name + ".bin").c_str(), "rb");
    if (!f) return v;
    std::fseek(f, 0, SEEK_END);
    const long bytes = std::ftell(f);
    std::fseek(f, 0, SEEK_SET);
    v.resize((size_t)bytes / sizeof(T));
    if (bytes > 0 && std::fread(v.data(), 1, (size_t)bytes, f) != (size_t)bytes) v.clear();
    std::fclose(f);
    return v;
}

int main(int argc, char **argv) {
    if (argc < 2) return 2;
    const std::string dir = argv[1];
    auto hdr = read_all<int64_t>(dir, "hdr");
    if (hdr.size() != 3) return 2;
    auto sp = read_all<int32_t>(dir, "succ_ptr"), si = read_all<int32_t>(dir, "succ_idx");
    auto st = read_all<int64_t>(dir, "succ_t");
    auto pp = read_all<int32_t>(dir, "pred_ptr"), pi = read_all<int32_t>(dir, "pred_idx");
    auto pe = read_all<int32_t>(dir, "pred_eid");
    auto c = read_all<int64_t>(dir, "c");
    auto lp = read_all<int32_t>(dir, "level_ptr"), lv = read_all<int32_t>(dir, "level_vtx");
    cpeval::Packed packed;
    const int rc = cpeval::pack_graph((int32_t)hdr[0], hdr[1], (int32_t)hdr[2], sp.data(), si.data(), st.data(),
                                      pp.data(), pi.data(), pe.data(), c.data(), lp.data(), lv.data(), packed);
    std::printf("rc=%d window=%d far_b=%d far_t=%d slots_b=%d blob=%zu\n", rc, (int)packed.have_window,
                packed.win_b.far_cap, packed.win_t.far_cap, packed.win_b.slots, packed.blob.size());
    return rc == 0 ? 0 : 1;
}
