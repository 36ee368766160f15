// Test helper (CPU only): the host-side lowering (grammar.cpp, tables.cpp) and the recogniser / accept cores, built with
// AddressSanitizer and UndefinedBehaviorSanitizer, run over inputs the test writes to files.  Not part of the library.
//   sanitize_main EBNF_FILE ROOT TOKENS_FILE SEQ_FILE
// TOKENS_FILE: per token a 4-byte little-endian length and the bytes; SEQ_FILE: int32 token ids (-1 ends a sequence).
#include <cstdint>
#include <cstdio>
#include <fstream>
#include <iterator>
#include <string>
#include <vector>

extern "C" long long xg2hc_check(const char* ebnf, size_t len, const char* root, const uint8_t* bytes, const uint64_t* offs, int n_tok,
                                 const uint8_t* sentence, size_t sentence_len, int max_contexts, char* msg, size_t msg_cap, long long* n_small_overflow);
extern "C" long long xg2hc_check_near(const char* ebnf, size_t len, const char* root, const uint8_t* bytes, const uint64_t* offs, int n_tok,
                                      char* msg, size_t msg_cap, long long* n_near, long long* max_depth);
extern "C" long long xg2hc_check_accept(const char* ebnf, size_t len, const char* root, const uint8_t* bytes, const uint64_t* offs, int n_tok,
                                        const int32_t* seq, int n_seq, const int32_t* try_ids, int n_try, int small_lists, char* msg, size_t msg_cap);

static std::string slurp(const char* path) {
    std::ifstream f(path, std::ios::binary);
    return std::string(std::istreambuf_iterator<char>(f), std::istreambuf_iterator<char>());
}

int main(int argc, char** argv) {
    if (argc != 5) { fprintf(stderr, "usage: sanitize_main EBNF ROOT TOKENS SEQ\n"); return 2; }
    const std::string ebnf = slurp(argv[1]), tok_file = slurp(argv[3]), seq_file = slurp(argv[4]);
    std::vector<uint8_t> bytes;
    std::vector<uint64_t> offs{0};
    for (size_t p = 0; p + 4 <= tok_file.size();) {
        uint32_t n = 0;
        for (int k = 0; k < 4; ++k) n |= (uint32_t)(uint8_t)tok_file[p + k] << (8 * k);
        p += 4;
        bytes.insert(bytes.end(), tok_file.begin() + (long)p, tok_file.begin() + (long)(p + n));
        p += n;
        offs.push_back(bytes.size());
    }
    bytes.push_back(0);
    std::vector<int32_t> seq(seq_file.size() / 4);
    for (size_t k = 0; k < seq.size(); ++k) {
        uint32_t v = 0;
        for (int b = 0; b < 4; ++b) v |= (uint32_t)(uint8_t)seq_file[4 * k + b] << (8 * b);
        seq[k] = (int32_t)v;
    }
    const int n_tok = (int)offs.size() - 1;
    char msg[512] = {0};
    long long small = 0, near = 0, deepest = 0;
    // the sentence for the recogniser check: the bytes of the first sequence
    std::vector<uint8_t> sentence;
    for (int32_t id : seq) { if (id < 0) break; sentence.insert(sentence.end(), bytes.begin() + (long)offs[(size_t)id], bytes.begin() + (long)offs[(size_t)id + 1]); }
    if (sentence.size() > 120) sentence.resize(120);
    const long long a = xg2hc_check(ebnf.data(), ebnf.size(), argv[2], bytes.data(), offs.data(), n_tok, sentence.data(), sentence.size(), 60, msg, sizeof msg, &small);
    if (a <= 0) { fprintf(stderr, "recogniser check: %s\n", msg); return 1; }
    const long long b = xg2hc_check_near(ebnf.data(), ebnf.size(), argv[2], bytes.data(), offs.data(), n_tok, msg, sizeof msg, &near, &deepest);
    if (b < 0) { fprintf(stderr, "near-equivalence check: %s\n", msg); return 1; }
    std::vector<int32_t> try_ids;
    for (int k = 1; k < n_tok && try_ids.size() < 6; k += 1 + n_tok / 7) try_ids.push_back(k);
    long long c = 0;
    for (int small_lists = 1; small_lists >= 0; --small_lists) {
        c = xg2hc_check_accept(ebnf.data(), ebnf.size(), argv[2], bytes.data(), offs.data(), n_tok, seq.data(), (int)seq.size(), try_ids.data(), (int)try_ids.size(),
                               small_lists, msg, sizeof msg);
        if (c <= 0) { fprintf(stderr, "accept check: %s\n", msg); return 1; }
    }
    printf("ok %lld %lld %lld\n", a, b, c);
    return 0;
}
