// placeholder until the dedicated temporal kernel lands
#include "ddit_common.hpp"
