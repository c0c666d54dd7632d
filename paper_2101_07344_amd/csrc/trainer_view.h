// What the serving side may see of a trainer: its shapes and the device addresses of its fp32 master
// weights (plain row-major).  Filled by train.hip, read by gati_cache_load_trainer in gati.hip.
#pragma once

struct gati_trainer;

namespace gati {

struct TrainerView {
    int device;
    int C;            // width of the trainer's input rows
    int H;            // first layer's outputs per position (0: no first layer)
    int K, Cin, P, Hin, Fsel;
    bool conv, sel_hidden_feat, no_selector;
    int Hs, Sx;       // hidden-layer selector: units, row stride of Ws (0: none)
    const float *W1, *b1, *W2, *b2, *ws, *bs, *Ws, *cs, *vs;
};

void trainer_view(const gati_trainer* t, TrainerView* v);

}  // namespace gati
