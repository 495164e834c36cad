// One translation unit per (element type, accumulator block count): compiled several times with
// -DDCNN_CONV_T=<f16|float> -DDCNN_CONV_TNAME=<f16|f32> -DDCNN_CONV_NB=<n> so the variants build in parallel.
#include "conv_impl.h"

#define DCNN_CAT_(a, b, c) launch_conv_##a##_nb##b
#define DCNN_CAT(a, b) DCNN_CAT_(a, b, 0)

namespace dcnn {

dcnn_status DCNN_CAT(DCNN_CONV_TNAME, DCNN_CONV_NB)(dcnn_ctx* ctx, bool init, const ListArgs& l, const ConvArgs& c,
                                                    const EpilogueArgs& e, const ConvPlan& p) {
    return launch_conv_nb<DCNN_CONV_T, DCNN_CONV_NB>(ctx, init, l, c, e, p);
}

}  // namespace dcnn
