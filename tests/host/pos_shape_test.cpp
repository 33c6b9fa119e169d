// Host-only check of the position-gather kernel's work-unit choice: prints one line per shape given on the
// command line (n h w c_in c_out k pad groups esize terms), or "no" when the layer is not eligible.
#include <cstdio>
#include <cstdlib>

#include "pos_shape.h"

int main(int argc, char** argv) {
    if (argc != 11) return 2;
    rrm_shape s{};
    s.kind = RRM_CONV;
    s.n = atoi(argv[1]); s.h = atoi(argv[2]); s.w = atoi(argv[3]); s.c_in = atoi(argv[4]); s.c_out = atoi(argv[5]);
    s.kh = s.kw = atoi(argv[6]); s.stride = 1; s.pad = atoi(argv[7]); s.groups = atoi(argv[8]);
    const int esize = atoi(argv[9]), terms = atoi(argv[10]);
    rrm::PosGeom g{};
    if (!rrm::pos_choose_shape(s, esize, terms, g)) {
        printf("no\n");
        return 0;
    }
    printf("G=%d R=%d RB=%d WP=%d npos=%d nbands=%d nsg=%d ncg=%d units=%d lds=%zu colcap=%d ts=%d nstage=%d nslab=%d\n", g.G, g.R,
           g.RB, g.WP, g.npos, g.nbands, g.nsg, g.ncg, g.total_units, rrm::conv_pos_lds_bytes(g, terms), g.col_cap, g.ts,
           g.nstage, g.nslab);
    return 0;
}
