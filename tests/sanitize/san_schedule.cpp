// Host sanitizer check of the schedule front end (parser, legality rules, lowering, search): the
// sources are compiled with this driver under -fsanitize=address,undefined and run on legal
// schedules, on mutants of them and on malformed text.  No device is touched.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "schedule.hpp"

namespace cst {
static std::string g_err;
void set_error(const char *fmt, ...) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_err = buf;
}
const char *get_error() { return g_err.c_str(); }
void clear_error() { g_err.clear(); }
}  // namespace cst

using namespace cst;

static int fails = 0;
static void expect(bool ok, const char *what) {
    if (!ok) { printf("FAIL: %s (%s)\n", what, get_error()); ++fails; }
}

static conststn_operand_desc csf_desc(const char *name, std::vector<int64_t> dims) {
    conststn_operand_desc d{};
    d.name = name;
    d.kind = CONSTSTN_OPERAND_CSF;
    d.csf = nullptr;
    d.order = int(dims.size());
    for (size_t i = 0; i < dims.size(); ++i) d.dims[i] = dims[i];
    return d;
}
static conststn_operand_desc dense_desc(const char *name, std::vector<int64_t> dims) {
    conststn_operand_desc d = csf_desc(name, dims);
    d.kind = CONSTSTN_OPERAND_DENSE;
    return d;
}

static conststn_status check(const char *text, const std::vector<conststn_operand_desc> &ops, const int *fusion = nullptr) {
    Schedule s;
    conststn_status st = parse_schedule(text, s);
    if (st != CONSTSTN_OK) return st;
    st = validate_schedule(s, fusion, int(ops.size()), ops.data());
    if (st == CONSTSTN_OK) (void)schedule_text(s);
    return st;
}

int main() {
    const std::vector<conststn_operand_desc> ttmc = {csf_desc("X", {9, 8, 7}), dense_desc("U3", {7, 4}), dense_desc("U2", {8, 3})};
    const char *ok = "T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s ; Y[i,r,s] = T[i,j,s] * U2[j,r] | i,j,r,s";
    expect(check(ok, ttmc) == CONSTSTN_OK, "legal TTMc schedule");
    const int f0[2] = {0, 0}, f3[2] = {3, 0};
    expect(check(ok, ttmc, f0) == CONSTSTN_OK, "unfused");
    expect(check(ok, ttmc, f3) == CONSTSTN_ESCHED, "fusion deeper than the common prefix");
    expect(check("T[i,j,s] = X[i,j,k] * U3[k,s] | j,i,k,s ; Y[i,r,s] = T[i,j,s] * U2[j,r] | i,j,r,s", ttmc) == CONSTSTN_ESCHED,
           "loop order against the level order");
    expect(check("Y[i,r,s] = T[i,j,s] * U2[j,r] | i,j,r,s ; T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s", ttmc) != CONSTSTN_OK,
           "consumer before producer");
    expect(check("T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k ; Y[i,r,s] = T[i,j,s] * U2[j,r] | i,j,r,s", ttmc) != CONSTSTN_OK,
           "loop list is not a permutation");
    const char *junk[] = {"", ";", "T[", "T[i] =", "T[i] = X[i,j,k]", "T[i] = X[i,j,k] *", "T[i] = X[i,j,k] * U3[k,s] |",
                          "T[i,,j] = X[i,j,k] * U3[k,s] | i,j,k,s", "= | ;;;", "T[i]=X[i]*X[i]|i;T[i]=X[i]*X[i]|i",
                          "T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s ; Y[i,r,s] = T[i,j,s] * Q[j,r] | i,j,r,s"};
    for (const char *t : junk) expect(check(t, ttmc) != CONSTSTN_OK, t);
    {   // very long names and many statements stay inside every buffer
        std::string name(300, 'n'), text = name + "[i] = X[i,j,k] * U3[k,s] | i,j,k,s";
        expect(check(text.c_str(), ttmc) == CONSTSTN_OK, "a 300-character tensor name");
        std::string many;
        for (int p = 0; p < 40; ++p) many += "T" + std::to_string(p) + "[i] = X[i,j,k] * U3[k,s] | i,j,k,s ;";
        (void)check(many.c_str(), ttmc);
    }
    // running example of the paper's Sec. 3.1 with its four sparse operands, and the search over the same tree
    const std::vector<conststn_operand_desc> abcd = {csf_desc("A", {4, 5, 6}), csf_desc("B", {7, 8, 4}), csf_desc("C", {7, 5, 9}),
                                                     csf_desc("D", {7, 8, 9})};
    (void)check("X[r,j,k] = B[r,l,i] * A[i,j,k] | r,j,k,l,i", abcd);
    {
        Schedule found;
        int l = 0;
        std::vector<std::vector<int>> modes;
        const conststn_status st = search_schedule("T[i,j,s] = X[i,j,k] * U3[k,s] ; Y[i,r,s] = T[i,j,s] * U2[j,r]", int(ttmc.size()),
                                                   ttmc.data(), false, 0, found, &l, modes);
        expect(st == CONSTSTN_OK && l >= 1, "search over the TTMc tree");
        expect(search_schedule("Y[i] = X[i,j,k] *", int(ttmc.size()), ttmc.data(), true, 0, found, &l, modes) != CONSTSTN_OK,
               "search refuses malformed trees");
    }
    printf("%s\n", fails ? "san_schedule: FAILED" : "san_schedule: ok");
    return fails ? 1 : 0;
}
