"""CPU oracle of the feature-extraction path.  Test infrastructure only: the
product package never imports anything from here."""
