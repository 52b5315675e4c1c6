// Driver for the sanitiser test: runs the host-only part of the library (packer, bin layout, work lists,
// E4M3 quantisers), built with -fsanitize=address,undefined, on cases read from a text file and writes every
// output as raw bytes, which the Python test compares with what the shipped library returns for the same
// cases.  Case lines:
//   pack <budget> <n> <lens...>
//   list <mask> <pass> <D> <Hq> <Hkv> <n> <lens...> <prefix words: 0, n or 2n of them>
//   quant <T> <H> <D> <seed>            per-head quantiser on pseudo-random bf16 bits
//   quantb <H> <D> <seed> <n> <lens...> block-wise quantiser
#include <cstdint>
#include <cstdio>
#include <fstream>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "../include/varlen_attn.h"

static void put(std::ofstream& out, const void* p, size_t bytes) { out.write(static_cast<const char*>(p), (std::streamsize)bytes); }
static void put_i32(std::ofstream& out, int32_t v) { put(out, &v, 4); }

// bf16 bit patterns of finite values of mixed magnitude (xorshift; exponent kept away from all-ones)
static std::vector<uint16_t> bf16_values(size_t n, uint32_t seed) {
    std::vector<uint16_t> x(n);
    uint32_t s = seed * 2654435761u + 1u;
    for (size_t i = 0; i < n; ++i) {
        s ^= s << 13;
        s ^= s >> 17;
        s ^= s << 5;
        const uint16_t sign = (uint16_t)((s >> 31) << 15);
        const uint16_t exp = (uint16_t)(110 + (s >> 8) % 30);  // 2^-17 .. 2^12
        const uint16_t man = (uint16_t)(s & 0x7f);
        x[i] = (uint16_t)(sign | (exp << 7) | man);
        if ((s >> 16) % 37 == 0) x[i] = 0;
    }
    return x;
}

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    std::ifstream in(argv[1]);
    std::ofstream out(argv[2], std::ios::binary);
    std::string line;
    while (std::getline(in, line)) {
        std::istringstream ls(line);
        std::string kind;
        ls >> kind;
        if (kind == "pack") {
            int32_t budget, n;
            ls >> budget >> n;
            std::vector<int32_t> lens((size_t)n), bin((size_t)n, -1), pos((size_t)n, -1);
            for (auto& v : lens) ls >> v;
            int32_t bins = -1;
            const int rc = va_pack_first_fit(lens.data(), n, budget, bin.data(), pos.data(), &bins);
            put_i32(out, rc);
            put_i32(out, bins);
            put(out, bin.data(), bin.size() * 4);
            put(out, pos.data(), pos.size() * 4);
        } else if (kind == "list") {
            int32_t mask, pass, D, Hq, Hkv, n;
            ls >> mask >> pass >> D >> Hq >> Hkv >> n;
            std::vector<int32_t> lens((size_t)n), prefix;
            for (auto& v : lens) ls >> v;
            int32_t w;
            while (ls >> w) prefix.push_back(w);
            std::vector<int32_t> cu((size_t)n + 1), pl((size_t)n);
            int32_t mx = -1;
            int rc = va_bin_layout(lens.data(), nullptr, n, cu.data(), nullptr, &mx);
            put_i32(out, rc);
            put(out, cu.data(), cu.size() * 4);
            size_t bytes = 0;
            rc = va_worklist_size(cu.data(), n, pass, D, Hq, Hkv, &bytes);
            put_i32(out, rc);
            if (rc != VA_OK) continue;
            std::vector<char> buf(bytes);  // exactly the size asked for: an overrun is the sanitiser's to find
            int32_t items = -1;
            rc = va_build_worklist(cu.data(), prefix.empty() ? nullptr : prefix.data(), n, mask, pass, D, Hq, Hkv, buf.data(),
                                   bytes, &items);
            put_i32(out, rc);
            put_i32(out, items);
            if (rc == VA_OK) put(out, buf.data(), bytes);
        } else if (kind == "quant") {
            int32_t T, H, D;
            uint32_t seed;
            ls >> T >> H >> D >> seed;
            const std::vector<uint16_t> x = bf16_values((size_t)T * H * D, seed);
            std::vector<uint8_t> codes(x.size());
            std::vector<float> descale((size_t)H);
            put_i32(out, va_quantize_e4m3_per_head(x.data(), T, H, D, codes.data(), descale.data()));
            put(out, x.data(), x.size() * 2);
            put(out, codes.data(), codes.size());
            put(out, descale.data(), descale.size() * 4);
        } else if (kind == "quantb") {
            int32_t H, D, n;
            uint32_t seed;
            ls >> H >> D >> seed >> n;
            std::vector<int32_t> cu((size_t)n + 1, 0);
            for (int32_t s = 0; s < n; ++s) {
                int32_t L;
                ls >> L;
                cu[(size_t)s + 1] = cu[(size_t)s] + L;
            }
            const int32_t T = cu[(size_t)n];
            const std::vector<uint16_t> x = bf16_values((size_t)T * H * D, seed);
            std::vector<uint8_t> codes(x.size());
            std::vector<float> descale((size_t)T * H);
            put_i32(out, va_quantize_e4m3_blockwise(x.data(), cu.data(), n, H, D, codes.data(), descale.data()));
            put(out, x.data(), x.size() * 2);
            put(out, codes.data(), codes.size());
            put(out, descale.data(), descale.size() * 4);
        } else if (!kind.empty()) {
            std::fprintf(stderr, "unknown case kind %s\n", kind.c_str());
            return 2;
        }
    }
    std::puts(va_last_error());
    return 0;
}
